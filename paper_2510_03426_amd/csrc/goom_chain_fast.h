// Hot variant of the chain kernel: float components, left factors given as GOOMs (or as real
// matrices) that fill the padded tile exactly (d = 16, 32, 64 or 128), state of 16 * NW columns;
// also, with the padding left out of the product, square sizes in between that are multiples of four.
// This is the kernel the long scans spend their time in (phase 1 and phase 3 of the
// three-phase scan; paper Section 4.1), and LMME on such shapes (Section 3.2).
// With BIAS one more wave carries column d of the augmented state [A* | b*] of a linear
// recurrence with bias (Section 4.3): it takes no part in converting the factor; its column is
// a matrix-vector product of the same LDS tile on the vector ALU (one row per lane, or per
// two or four lanes), to which it adds the step's bias vector.
//
// On this chip the float matrix instructions run at the rate of the vector ALU and do
// not overlap with it, so a step costs (matrix cycles) + 4 x (vector instructions) and
// the design goal is to spend as few vector instructions per element as possible:
//   * a lane loads four adjacent elements (two 16-byte loads), so a row's maximum needs
//     three local and log2(lanes per row) cross-lane integer maxima on the vector ALU;
//   * exponentiation is two fused multiply-adds and one hardware exp2 per element; the
//     sign is the parity bit of round(im / pi) moved onto the sign bit;
//   * the running product is NOT rescaled after a step.  The row exponents n_i that the
//     step leaves behind are folded into the exponent arguments of the next factor's
//     columns instead (the next product contracts over exactly those rows), which costs
//     one subtraction per element there and nothing here.  Columns are renormalised by a
//     power of two every few steps only, to stay inside float range;
//   * output addresses are lane base + compile-time offsets.
#pragma once
#include "goom_chain_kernel.h"

namespace goom_chain {

struct Item4 {
    f4 a, b; // (re0, im0, re1, im1), (re2, im2, re3, im3)
};

__device__ inline float vmax_raw(float x, float y)
{
    // plain v_max_f32: the compiler's own max first canonicalises both operands
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(y));
    return r;
}

template <int CTRL> __device__ inline float add_dpp(float x)
{
    const int y = __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true);
    return x + __builtin_bit_cast(float, y);
}

// REAL: the left factors are plain real matrices (4 bytes per entry instead of a GOOM's 8): an entry is
// scaled by 2^(r_j - n_i) exactly, with no logarithm or exponential on the way in.
// RAG: square matrices of a size d < DP that is a multiple of four (rows d entries apart in memory): the
// tile's rows and columns from d on are zero, only the first KD = ceil(d / 16) blocks of sixteen rows and
// columns take part in the product, and waves whose sixteen state columns lie beyond d only help converting.
template <int DP, int NW, bool BIAS, bool REAL, int KD = DP / 16, bool RAG = false>
__device__ __forceinline__ void chain_body(const ChainArgs &a)
{
    typedef Comp<float> C;
    static_assert(!RAG || (!BIAS && !REAL && KD <= DP / 16), "ragged sizes: GOOM factors, no bias column");
    constexpr int KT = KD;
    constexpr int LDA = DP + 4;
    constexpr int NWT = NW + (BIAS ? 1 : 0); // waves, one per 16-column slab of the state
    constexpr int M = 16 * NWT;  // state columns
    constexpr int NT = NW * 64;  // threads that convert the factor
    constexpr int LPR = DP / 4;  // lanes per row of the factor
    constexpr int NITEMS = DP * LPR;
    constexpr int Q = NITEMS / NT; // items per thread
    constexpr int kRenormEvery = 4;
    static_assert(NITEMS % NT == 0 && NT % LPR == 0, "tile does not divide among the threads");
    // A pass of all converting threads covers NT / LPR rows of the factor.  Ragged sizes: that is sixteen rows,
    // so only the first KD passes hold rows that take part in the product; the others are neither loaded nor
    // converted (their row exponents, those of zero rows, are written once at the start).
    static_assert(!RAG || (NT / LPR == 16 && Q == DP / 16), "ragged sizes: one pass per block of sixteen rows");
    constexpr int QE = RAG ? KD : Q;
    constexpr size_t kTileBytes = (size_t)DP * LDA * sizeof(float);
    constexpr size_t kBufBytes = kTileBytes + (size_t)DP * sizeof(float);

    extern __shared__ __align__(16) unsigned char smem[];
    auto tile_of = [&](int b) { return reinterpret_cast<float *>(smem + (size_t)b * kBufBytes); };
    auto nsh_of = [&](int b) { return reinterpret_cast<float *>(smem + (size_t)b * kBufBytes + kTileBytes); };
    double *wave_red = reinterpret_cast<double *>(smem + 2 * kBufBytes);
    float *wvec = reinterpret_cast<float *>(smem + 2 * kBufBytes + 128); // the bias wave's column (BIAS only)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4;
    const int c = lane & 15;
    const int col = wave * 16 + c;
    const int c4 = 4 * (tid % LPR); // first of this lane's four factor columns
    const bool converter = !BIAS || wave < NW;
    const bool bias_wave = BIAS && wave == NW;
    const int dd = RAG ? a.d : DP;        // size of the matrices in memory
    // this wave owns sixteen columns of the state (KD may exceed ceil(d / 16) when a wider state elsewhere in
    // the same scan has fixed the tile size; the factored product stored at the end has ceil(d / 16) slabs)
    const bool owner = !RAG || (wave < KD && 16 * wave < dd);
    // bias wave: lane -> row and part of the contraction index
    constexpr int LPRB = DP >= 64 ? 1 : 64 / DP; // lanes per row
    constexpr int CPLB = DP / LPRB;              // contraction indices per lane
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

    auto load_items = [&](long long t, Item4 (&it)[Q]) {
        const float *src = reinterpret_cast<const float *>(left0 + t * a.left_step_stride);
#pragma unroll
        for (int q = 0; q < QE; ++q) {
            const int row = (tid + q * NT) / LPR;
            if (REAL) {
                it[q].a = *reinterpret_cast<const f4 *>(src + (size_t)row * DP + c4);
            } else if (RAG) {
                // entries beyond the matrix are read from its last row / last four columns instead (and
                // discarded by the conversion), so that no load sits behind a branch
                const int rr = row < dd ? row : dd - 1, cc = c4 < dd ? c4 : dd - 4;
                const f4 *gp = reinterpret_cast<const f4 *>(src + ((size_t)rr * dd + cc) * 2);
                it[q].a = gp[0];
                it[q].b = gp[1];
            } else {
                const f4 *gp = reinterpret_cast<const f4 *>(src + ((size_t)row * DP + c4) * 2);
                it[q].a = gp[0];
                it[q].b = gp[1];
            }
        }
    };

    // tile[i][j] = (+-) 2^(log2|A_ij| + r_j - n_i),  n_i = ceil(max_j (log2|A_ij| + r_j)),
    // r_j = row exponents still attached to the running product (zero at the start).
    auto convert_items = [&](const Item4 (&it)[Q], int buf, const float *rsrc) {
        const float kHi = 1.44269502162933349609375f; // float nearest log2(e)
        const float kLo = 1.925963033500011e-8f;      // log2(e) - kHi
        float *tile = tile_of(buf);
        float *nsh = nsh_of(buf);
        f4 rj = {0.f, 0.f, 0.f, 0.f};
        // (ragged: columns beyond the matrix carry the exponent of a zero row, which the rows beyond the
        // matrix hand on from step to step; it makes their entries vanish)
        if (RAG && c4 >= dd) rj = f4{-1.0e30f, -1.0e30f, -1.0e30f, -1.0e30f};
        if (rsrc) rj = *reinterpret_cast<const f4 *>(&rsrc[c4]);
#pragma unroll
        for (int q = 0; q < QE; ++q) {
            const int row = (tid + q * NT) / LPR;
            if (REAL) {
                // binary exponents (frexp convention) take the place of the log2 magnitudes, in integer
                // arithmetic throughout; all shifts are exact.  (A zero entry counts as exponent 0: the row
                // shift only has to be large enough, and scaling by a power of two loses nothing.)
                int rji[4], ei[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    rji[e] = (int)rj[e]; // row exponents are whole numbers
                    ei[e] = __builtin_amdgcn_frexp_expf(it[q].a[e]) + rji[e];
                }
                int key = C::imax(C::imax(ei[0], ei[1]), C::imax(ei[2], ei[3]));
                key = C::imax(key, C::dpp<0xB1>(key));
                if (LPR >= 4) key = C::imax(key, C::dpp<0x4E>(key));
                if (LPR >= 8) key = C::imax(key, C::dpp<0x141>(key));
                if (LPR >= 16) key = C::imax(key, C::dpp<0x140>(key));
                if (LPR >= 32) key = C::xor16_imax(key);
                f4 y;
#pragma unroll
                for (int e = 0; e < 4; ++e) y[e] = __builtin_ldexpf(it[q].a[e], rji[e] - key);
                *reinterpret_cast<f4 *>(&tile[row * LDA + c4]) = y;
                nsh[row] = (float)key;
                continue;
            }
            const float re[4] = {it[q].a[0], it[q].a[2], it[q].b[0], it[q].b[2]};
            const float im[4] = {it[q].a[1], it[q].a[3], it[q].b[1], it[q].b[3]};
            // row maximum of log2|A_ij| + r_j, to within rounding (any nearby whole number serves)
            float u = __builtin_fmaf(re[0], kHi, rj[0]);
#pragma unroll
            for (int e = 1; e < 4; ++e) u = vmax_raw(u, __builtin_fmaf(re[e], kHi, rj[e]));
            int key = C::key_of(u);
            key = C::imax(key, C::dpp<0xB1>(key));
            if (LPR >= 4) key = C::imax(key, C::dpp<0x4E>(key));
            if (LPR >= 8) key = C::imax(key, C::dpp<0x141>(key));
            if (LPR >= 16) key = C::imax(key, C::dpp<0x140>(key));
            if (LPR >= 32) key = C::xor16_imax(key);
            float mx = C::of_key(key);
            // a row that is entirely zero keeps a finite (hugely negative) shift, and its
            // exponent arguments are forced to -inf so that nothing can overflow
            const bool zero_row = !(mx > -1.0e30f) || (RAG && row >= dd);
            // (with a bias column the shift of such a row must stay small: the bias is scaled by it)
            const float n = zero_row ? (BIAS ? 0.0f : -1.0e30f) : __builtin_ceilf(mx);
            const float nsub = zero_row ? __builtin_huge_valf() : n;
            f4 y;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // exponent argument with one rounding at its own (small) magnitude, then the low part of log2(e)
                float t = __builtin_fmaf(re[e], kHi, rj[e] - nsub);
                t = __builtin_fmaf(re[e], kLo, t);
                const float v = __builtin_amdgcn_exp2f(t); // 2^-inf = 0 covers zero entries
                // parity of round(im / pi), read off the last mantissa bit after adding 1.5 * 2^23, and put on the sign
                // bit with one shift-and-or (v is an exponential: its own sign bit is clear)
                const float kf = __builtin_fmaf(im[e], 0.318309886183790671538f, 12582912.0f);
                y[e] = __builtin_bit_cast(float, __builtin_bit_cast(int, v) | (__builtin_bit_cast(int, kf) << 31));
            }
            *reinterpret_cast<f4 *>(&tile[row * LDA + c4]) = y;
            nsh[row] = n; // every lane of the row writes the same value
        }
    };

    // ------------------------------------------------------------------ initial state
    float st[KT][4]; // st[kt][v] = W[16 kt + 4 g + v][col]
    double ecol = 0.0;
    const size_t fact_mant_bytes = (size_t)DP * a.fact_cols * sizeof(float);
    if (a.init_mode == 0 || a.init_mode == 3) {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) st[kt][v] = (a.init_mode == 0 && 16 * kt + 4 * g + v == col && col < dd) ? 1.0f : 0.0f;
    } else if (!owner) {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) st[kt][v] = 0.0f;
    } else if (a.init_mode == 1) {
        long long iidx = chain_global;
        if (a.init_group > 0) {
            long long grp = chunk / a.init_group;
            if (grp >= a.init_ngroups) grp = a.init_ngroups - 1;
            iidx = (item * a.init_ngroups + grp) * (a.init_group + 1) + (chunk - grp * a.init_group);
        }
        const unsigned char *ip = a.init + iidx * a.init_stride;
        const float *mp = reinterpret_cast<const float *>(ip);
        const double *ep = reinterpret_cast<const double *>(ip + fact_mant_bytes);
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) st[kt][v] = mp[(size_t)(16 * kt + 4 * g + v) * a.fact_cols + col];
        ecol = ep[col];
    } else {
        const float *gp = reinterpret_cast<const float *>(a.init + item * a.init_stride);
        const int MM = RAG ? dd : M; // columns of the initial state in memory
        // (ragged: entries beyond the matrix are read from its last row / column and replaced by zeros)
        const int colc = RAG ? (col < dd ? col : dd - 1) : col;
        auto init_row = [&](int r) { return RAG ? (r < dd ? r : dd - 1) : r; };
        auto init_ok = [&](int r) { return !RAG || (r < dd && col < dd); };
        float cmax = C::neg_inf();
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int r = 16 * kt + 4 * g + v;
                const float re = gp[((size_t)init_row(r) * MM + colc) * 2];
                cmax = C::max_(cmax, init_ok(r) ? re : C::neg_inf());
            }
        cmax = C::xor16_32_max(cmax);
        // the column's exponent: a whole number near its largest log2 magnitude that a float holds exactly
        const float ecol_f = (cmax > C::neg_inf()) ? (float)__builtin_ceil((double)cmax * kLog2e) : 0.0f;
        ecol = (double)ecol_f;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int r = 16 * kt + 4 * g + v;
                const float2 e = *reinterpret_cast<const float2 *>(gp + ((size_t)init_row(r) * MM + colc) * 2);
                st[kt][v] = init_ok(r) ? C::apply_sign(C::exp2_shifted(e.x, ecol_f), e.y) : 0.0f;
            }
    }

    Item4 pre[Q];
    if (RAG) {
        for (int i = 16 * KD + tid; i < DP; i += NT) nsh_of(0)[i] = nsh_of(1)[i] = -1.0e30f;
    }
    if (len > 0 && converter) {
        load_items(0, pre);
        convert_items(pre, 0, nullptr);
        if (len > 1) load_items(1, pre);
    }
    // bias wave: entry brow of a step's bias vector, and its column of the state (also kept in LDS,
    // where the lanes read the entries they contract over); the column starts at zero
    float2 bpre = {0.0f, 0.0f};
    auto load_bias = [&](long long t) {
        bpre = *reinterpret_cast<const float2 *>(a.bias + ((size_t)(item * a.steps + t0 + t) * DP + brow) * 8);
    };
    if (BIAS && bias_wave && lane < DP) wvec[lane] = 0.0f;
    if (BIAS && bias_wave && len > 0) load_bias(0);
    __syncthreads();

    for (long long t = 0; t < len; ++t) {
        const int cur = (int)(t & 1);
        const float *tile = tile_of(cur);
        const float *nsh = nsh_of(cur);
        const bool last = t == len - 1;

        // ------------------------------------------------------------ product, and next factor beside it
        f4 acc[KT];
        float accb = 0.0f;
        if (BIAS && bias_wave) {
            // column d of the product: row brow of the tile times the column, on the vector ALU
#pragma unroll
            for (int k = 0; k < CPLB / 4; ++k) {
                const f4 av = *reinterpret_cast<const f4 *>(&tile[brow * LDA + bc0 + 4 * k]);
                const f4 wv = *reinterpret_cast<const f4 *>(&wvec[bc0 + 4 * k]);
#pragma unroll
                for (int e = 0; e < 4; ++e) accb = __builtin_fmaf(av[e], wv[e], accb);
            }
            if (LPRB >= 2) accb = add_dpp<0xB1>(accb);
            if (LPRB >= 4) accb = add_dpp<0x4E>(accb);
        } else if (owner) {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) acc[mt] = f4{0, 0, 0, 0};
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                f4 av[KT];
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
                    av[mt] = *reinterpret_cast<const f4 *>(&tile[(16 * mt + c) * LDA + 16 * kt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int mt = 0; mt < KT; ++mt) acc[mt] = C::mfma(av[mt][v], st[kt][v], acc[mt]);
            }
        }
        // (after the last product there is nothing to convert: a single product, as in a
        // batched LMME, would otherwise pay for its left factor twice)
        if (converter && !last) {
            convert_items(pre, cur ^ 1, nsh);
            load_items(t + 2 < len ? t + 2 : len - 1, pre);
        }
        float nrb = 0.0f;
        if (BIAS && bias_wave) {
            // b_i enters entry (i, d) of the product, which is held as accb 2^(n_i + ecol): add
            // (+-) 2^(log2|b_i| - n_i - ecol).  Should the column have shrunk so far below the bias
            // that this would overflow, the column is first scaled down (to nothing, if need be).
            const float kHi = 1.44269502162933349609375f;
            const float kLo = 1.925963033500011e-8f;
            nrb = nsh[brow];
            if (__builtin_amdgcn_ballot_w64(accb != 0.0f) == 0) {
                // a zero column has no scale of its own: it takes the bias's, whatever its magnitude
                float m = __builtin_fmaf(bpre.x, kHi, -nrb);
                m = C::template group_allmax<64>(m, m);
                ecol = (m > -1.0e30f && m < 1.0e30f) ? (double)__builtin_ceilf(m) : 0.0;
            }
            float x = __builtin_fmaf(bpre.x, kHi, -(nrb + (float)ecol));
            x = __builtin_fmaf(bpre.x, kLo, x);
            float down = 0.0f;
            if (__builtin_amdgcn_ballot_w64(x > 64.0f) != 0) {
                const float amax = C::template group_allmax<64>(x, x);
                down = C::max_(0.0f, __builtin_ceilf(amax) - 64.0f);
                accb = __builtin_ldexpf(accb, -(int)C::clamp_shift(down));
                ecol += (double)down;
            }
            accb += C::apply_sign(__builtin_amdgcn_exp2f(x - down), bpre.y);
            load_bias(t + 1 < len ? t + 1 : len - 1);
        }

        // ------------------------------------------------------------ outputs
        // entry (i = 16 mt + 4 g + v, col) of the product is acc 2^(n_i + ecol)
        const bool want_out = a.out_goom && (!a.out_goom_last_only || last) && !bias_wave && owner;
        if (want_out && !RAG) {
            const long long o_idx = a.out_goom_last_only ? chain_global : (item * a.steps + t0 + t);
            float *outp = reinterpret_cast<float *>(a.out_goom) + ((size_t)o_idx * DP * M + (size_t)(4 * g) * M + col) * 2;
            const float ecol_f = (float)ecol;
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                const f4 nv = *reinterpret_cast<const f4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float x = acc[mt][v];
                    const float re = C::out_re_f(x, nv[v] + ecol_f);
                    const float im = x < 0.0f ? C::pi() : 0.0f;
                    *reinterpret_cast<float2 *>(outp + (size_t)(16 * mt + v) * M * 2) = float2{re, im};
                }
            }
        }
        if (want_out && RAG) {
            // rows d entries apart; a lane's four rows 16 mt + 4 g + v lie inside the matrix together (d is a
            // multiple of four)
            const long long o_idx = a.out_goom_last_only ? chain_global : (item * a.steps + t0 + t);
            float *outp = reinterpret_cast<float *>(a.out_goom) + ((size_t)o_idx * dd * dd + (size_t)(4 * g) * dd + col) * 2;
            const float ecol_f = (float)ecol;
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                if (16 * mt + 4 * g < dd && col < dd) {
                    const f4 nv = *reinterpret_cast<const f4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float x = acc[mt][v];
                        const float re = C::out_re_f(x, nv[v] + ecol_f);
                        const float im = x < 0.0f ? C::pi() : 0.0f;
                        *reinterpret_cast<float2 *>(outp + (size_t)(16 * mt + v) * dd * 2) = float2{re, im};
                    }
                }
            }
        }

        // ------------------------------------------------------------ state for the next step
        if (BIAS && bias_wave) {
            // the same bookkeeping for the one column: raw between steps, renormalised now and then,
            // row exponents folded in at the end
            if (!last) {
                if ((t % kRenormEvery) == kRenormEvery - 1) {
                    float cm = C::max_(-300.0f, C::exponent_of(accb));
                    cm = C::template group_allmax<64>(cm, cm);
                    accb = __builtin_ldexpf(accb, -(int)cm);
                    ecol += (double)cm;
                }
            } else {
                float cm = C::exponent_of(accb) + nrb;
                cm = C::template group_allmax<64>(cm, cm);
                accb = __builtin_ldexpf(accb, (int)C::clamp_shift(nrb - cm));
                ecol += (double)cm;
            }
            if (lane % LPRB == 0) wvec[brow] = accb;
        } else if (!owner) {
            // (no state columns)
        } else if (!last) {
            // keep the raw product; its row exponents n_i go to the next factor's columns
#pragma unroll
            for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v) st[mt][v] = acc[mt][v];
            if ((t % kRenormEvery) == kRenormEvery - 1) {
                float cm = -300.0f;
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) cm = C::max_(cm, C::exponent_of(st[mt][v]));
                cm = C::xor16_32_max(cm);
                const int sh = -(int)cm;
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) st[mt][v] = __builtin_ldexpf(st[mt][v], sh);
                ecol += (double)cm;
            }
        } else {
            // last step: fold the row exponents into the mantissas, one exponent per column
            float cm = C::neg_inf();
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                const f4 nv = *reinterpret_cast<const f4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v) cm = C::max_(cm, C::exponent_of(acc[mt][v]) + nv[v]);
            }
            cm = C::xor16_32_max(cm);
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                const f4 nv = *reinterpret_cast<const f4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    st[mt][v] = __builtin_ldexpf(acc[mt][v], (int)C::clamp_shift(nv[v] - cm));
            }
            ecol += (double)cm;
        }
        __syncthreads();
    }

    if (a.out_fact_final) {
        // factored product of the chain, all columns on one exponent (it becomes a left factor)
        unsigned char *dst = a.out_fact_final + chain_global * a.fact_stride;
        float *mp = reinterpret_cast<float *>(dst);
        double *ep = reinterpret_cast<double *>(dst + fact_mant_bytes);
        float cm = 0.0f;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) cm = C::max_(cm, __builtin_fabsf(st[kt][v]));
        cm = C::xor16_32_max(cm);
        // (the bias column is not contracted over when the product serves as a left factor: it
        // keeps an exponent of its own, so a bias far above or below A* costs neither any bits)
        double ev = (cm > 0.0f && !bias_wave && owner) ? ecol : kNegBig;
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
        const int shift = (cm > 0.0f && !bias_wave) ? (int)dsh : 0;
        if (BIAS && bias_wave) {
            // column d from the lanes that own its rows; the padding columns behind it are zero
            if (lane % LPRB == 0) mp[(size_t)brow * a.fact_cols + DP] = wvec[brow];
            for (int idx = lane; idx < DP * 15; idx += 64) mp[(size_t)(idx / 15) * a.fact_cols + DP + 1 + idx % 15] = 0.0f;
        } else if (owner) {
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    mp[(size_t)(16 * kt + 4 * g + v) * a.fact_cols + col] = __builtin_ldexpf(st[kt][v], shift);
        }
        if (g == 0 && owner) ep[col] = bias_wave ? ecol : emax;
    }
}

// (second launch bound: waves per SIMD the register allocation has to leave room for)
template <int DP, int NW, bool BIAS>
__global__ __launch_bounds__((NW + (BIAS ? 1 : 0)) * 64, (DP <= 16 ? 8 : DP == 32 ? (BIAS ? 5 : 6) : DP == 64 ? (BIAS ? 3 : 4) : 2)) void chain_kernel_fast(ChainArgs a)
{
    chain_body<DP, NW, BIAS, false>(a);
}

template <int DP, int NW>
__global__ __launch_bounds__(NW * 64, (DP <= 16 ? 8 : DP == 32 ? 6 : DP == 64 ? 4 : 2)) void chain_kernel_fast_real(ChainArgs a)
{
    chain_body<DP, NW, false, true>(a);
}

// square matrices of a size below DP (a multiple of four), KD = ceil(d / 16) blocks of sixteen
template <int DP, int NW, int KD>
__global__ __launch_bounds__(NW * 64, (DP == 32 ? 6 : DP == 64 ? 4 : 2)) void chain_kernel_fast_ragged(ChainArgs a)
{
    chain_body<DP, NW, false, false, KD, true>(a);
}

template <int DP, int NW, bool BIAS, bool REAL = false> int launch_fast(goom_ctx *ctx, const ChainArgs &args, long long grid, const char *label)
{
    constexpr int LDA = DP + 4;
    const size_t lds = 2 * ((size_t)DP * LDA * sizeof(float) + (size_t)DP * sizeof(float)) + 128 + (BIAS ? DP * sizeof(float) : 0);
    void (*kern)(ChainArgs);
    if constexpr (REAL) kern = chain_kernel_fast_real<DP, NW>;
    else kern = chain_kernel_fast<DP, NW, BIAS>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return goom::check_hip(ctx, e, "hipFuncSetAttribute(chain_kernel_fast)");
    }
    if (grid <= 0) return GOOM_OK;
    if (grid > 0x7fffffffLL) return goom::fail(ctx, GOOM_EUNSUPPORTED, "too many chains for one launch (%lld)", grid);
    goom::prof_begin(ctx, label);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3((NW + (BIAS ? 1 : 0)) * 64), lds, ctx->stream, args);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch chain_kernel_fast");
}

// The hot variant applies when the factor fills its padded tile, every wave owns a full
// slab, there is no bias, and no per-step factored output is wanted.
inline bool fast_applies(const ChainArgs &args, int dp, int nw)
{
    return args.n == dp && args.d == dp && args.m == 16 * nw && args.bias_mode == 0 && args.out_fact_steps == nullptr &&
           ((dp == 16 && nw == 1) || (dp == 32 && nw == 2) || (dp == 64 && nw == 4) || (dp == 128 && nw == 8)) &&
           (!args.left_real || dp >= 32);
}

// Kernels of the linear recurrence with bias (separate translation unit): chunk products of
// the augmented matrices with the extra bias wave, and the matrix-vector walk that produces
// the states from the carried vectors.
bool affine_chunk_applies(const ChainArgs &args, int dp);
int dispatch_affine_chunk(goom_ctx *ctx, const ChainArgs &args, int dp, long long grid, const char *label);
bool affine_walk_applies(const ChainArgs &args, int dp);
int dispatch_affine_walk(goom_ctx *ctx, const ChainArgs &args, int dp, long long grid, const char *label);
int launch_replicate_power(goom_ctx *ctx, void *totals, long long stride, int fact_cols, int dp, int d, long long batch,
                           long long chunks, long long chunks_per_item, bool f64);
int dispatch_affine_chunk_f64(goom_ctx *ctx, const ChainArgs &args, int dp, long long grid, const char *label);

// square matrices whose size is a multiple of four between the sizes above (20 ... 124): the hot kernel
// with the rows and columns beyond the matrix left out, separate translation unit
bool ragged_applies(const ChainArgs &args, int dp, int nw);
int dispatch_ragged(goom_ctx *ctx, const ChainArgs &args, int dp, long long grid, const char *label);

// 8 x 8 and 16 x 16 chains: one wave per chain (or per pair of 8 x 8 chains), separate translation unit
bool small_applies(const ChainArgs &args, int dp);
int dispatch_small(goom_ctx *ctx, const ChainArgs &args, long long nchains, const char *label);

inline int dispatch_fast(goom_ctx *ctx, const ChainArgs &args, int dp, long long grid, const char *label)
{
    if (args.left_real) {
        switch (dp) {
        case 32: return launch_fast<32, 2, false, true>(ctx, args, grid, label);
        case 64: return launch_fast<64, 4, false, true>(ctx, args, grid, label);
        default: return launch_fast<128, 8, false, true>(ctx, args, grid, label);
        }
    }
    switch (dp) {
    case 16: return launch_fast<16, 1, false>(ctx, args, grid, label);
    case 32: return launch_fast<32, 2, false>(ctx, args, grid, label);
    case 64: return launch_fast<64, 4, false>(ctx, args, grid, label);
    default: return launch_fast<128, 8, false>(ctx, args, grid, label);
    }
}

} // namespace goom_chain
