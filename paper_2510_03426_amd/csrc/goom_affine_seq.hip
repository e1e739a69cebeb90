// Linear recurrence with bias, h_t = A_t h_{t-1} + b_t over GOOMs (paper Section 4.3), float components, d = 32, for
// batches of many sequences: one workgroup walks one whole sequence, step after step, and reads every matrix once.
//
// With a hundred sequences or more there is no need to cut a sequence into chunks (whose products cost a matrix-matrix
// product per step and a second pass over the matrices): a workgroup keeps twelve steps of its sequence's matrices in
// flight, which is enough outstanding memory traffic per compute unit, and a step is a matrix-vector product.  The
// work of a step falls into a part that does not depend on the running vector and a chain that does, and the
// waves of the workgroup are split accordingly, one wave of each kind per SIMD, so that the first fills the waits of
// the second; a ninth wave writes the states out:
//
//   * waves 0-3 scale the matrices, one step ahead: a lane loads four adjacent entries of a row (eight lanes a row,
//     eight rows a wave), the row's lanes agree on its power-of-two shift n_i, and (+-) 2^(log2|A_ij| - n_i) goes to
//     LDS with n_i and with what the chain needs of the row's bias (a whole-number exponent at or above its log2
//     magnitude, its log-magnitude, its sign bit);
//   * waves 4-7 run the chain: the vector lives in LDS as float mantissas with one whole-number exponent per group of
//     eight entries (the rows one wave produces); a lane reads four scaled entries of its row and its four entries of
//     the vector, brings these to the largest group exponent G, and the row's eight lanes add up their products: entry
//     i of A_t h is that sum times 2^(n_i + G).  The bias b_i joins on the new exponent of the wave's eight rows (the
//     largest of the eight sums' and the eight bias terms' exponents), the wave writes eight mantissas and that exponent.
//
// One workgroup barrier ends a step: scaled matrices, mantissas and exponents alternate between two sets of LDS words.
// The state of step t - 1 leaves during step t, through wave 8: as a GOOM, and / or as the scaled exponential of Section 4.3, eq. 27
// with its log-scaling constant.  Nothing but A_t, b_t (read once) and the outputs (written once) touches HBM; the chain
// waves touch no memory but LDS.
#include "goom_chain_fast.h"
#include <type_traits>

namespace goom_chain {

namespace {

constexpr int kSeqDepth = 8;          // steps written out per round of the chain waves' loop
constexpr int kSeqRing = 12;          // steps of a sequence in flight (forward)
constexpr int kSeqRingAdj = 10;       // ... adjoint recurrence (one register more per step and lane)
constexpr int kSeqNone = -(1 << 28);  // exponent of a group of zeros
constexpr int kSeqExpLimit = 1 << 27; // whole-number exponents are kept inside +- this
constexpr int kSeqD = 32;
constexpr int kSeqThreads = 9 * 64;    // four waves for the matrices, four for the chain, one for the outputs

struct SeqArgs {
    const unsigned char *A;    // [batch, T, 32, 32] complex64
    const unsigned char *bias; // [batch, T, 32] complex64
    const unsigned char *h0;   // NULL (zero) or [batch, 32] complex64
    unsigned char *out_goom;   // NULL or [batch, T, 32] complex64
    float *out_scaled;         // NULL or [batch, T, 32]
    float *out_logscale;       // NULL or [batch, T]
    const float *left_shift;   // adjoint recurrence only: [batch, T] floats (see ChainArgs::left_shift)
    long long T;
};

struct SeqShared {
    float sv[2][kSeqD * (kSeqD + 1)]; // scaled, signed entries of a step's matrix (adjoint recurrence: rows one word apart more, read by columns)
    int nsrc[2][kSeqD];               // adjoint recurrence: the row shifts of the matrix as stored (they go with the vector's entries)
    int4 rec[2][kSeqD];         // per row: its shift n_i; the bias's whole-number exponent, log-magnitude (float bits) and sign bit
    float m[2][kSeqD];          // mantissas of the vector
    int f[2][4];                // exponent of entries 8 w .. 8 w + 7 (the rows chain wave w produces)
};

// Workgroup barrier that orders LDS traffic only: the matrices in flight from HBM stay in flight across it (the
// general barrier would wait for every outstanding load, and with it for the whole ring of prefetched steps).
__device__ inline void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// The rings of prefetched steps: loads the compiler does not track (it would make every step wait for the loads issued in it,
// to copy what they fetched to the registers of the step that consumes it), issued and awaited by hand.  A load's registers
// pass through the wait before their first use, so nothing reads them earlier; a wave's vector-memory loads return in the
// order of issue, and stores issued in between only make the wait stricter.
typedef float f2 __attribute__((ext_vector_type(2)));
__device__ inline void load_matrix_part(f4 &x, f4 &y, f2 &b, const unsigned char *p, const unsigned char *pb)
{
    asm volatile("global_load_dwordx4 %0, %3, off\n\tglobal_load_dwordx4 %1, %3, off offset:16\n\tglobal_load_dwordx2 %2, %4, off"
                 : "=&v"(x), "=&v"(y), "=&v"(b)
                 : "v"(p), "v"(pb)
                 : "memory");
}
// the same with the step's shift (adjoint recurrence)
__device__ inline void load_matrix_part_shift(f4 &x, f4 &y, f2 &b, float &sh, const unsigned char *p, const unsigned char *pb, const float *ps)
{
    asm volatile("global_load_dwordx4 %0, %4, off\n\tglobal_load_dwordx4 %1, %4, off offset:16\n\tglobal_load_dwordx2 %2, %5, off\n\t"
                 "global_load_dword %3, %6, off"
                 : "=&v"(x), "=&v"(y), "=&v"(b), "=&v"(sh)
                 : "v"(p), "v"(pb), "v"(ps)
                 : "memory");
}
// what was issued kSeqDepth steps ago has landed once at most NEWER younger loads are outstanding
template <int NEWER> __device__ inline void wait_matrix_part_shift(f4 &x, f4 &y, f2 &b, float &sh)
{
    asm volatile("s_waitcnt vmcnt(%4)" : "+v"(x), "+v"(y), "+v"(b), "+v"(sh) : "n"(NEWER) : "memory");
}
template <int NEWER> __device__ inline void wait_matrix_part(f4 &x, f4 &y, f2 &b) { asm volatile("s_waitcnt vmcnt(%3)" : "+v"(x), "+v"(y), "+v"(b) : "n"(NEWER) : "memory"); }

template <int I, int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

constexpr float kSeqHi = 1.44269502162933349609375f; // float nearest log2(e)
constexpr float kSeqLo = 1.925963033500011e-8f;      // log2(e) - kSeqHi

// whole-number exponent at or above log2 of a magnitude given by its natural logarithm; kSeqNone for a zero
__device__ inline int exponent_above(float re)
{
    const float e = __builtin_amdgcn_fmed3f(__builtin_ceilf(re * kSeqHi), -(float)kSeqExpLimit, (float)kSeqExpLimit);
    return re > -__builtin_huge_valf() ? (int)e : kSeqNone;
}
// (+-) 2^(re log2(e) - f) for a whole number f, the product with log2(e) carried in two floats
__device__ inline float scaled_term(float re, float im, int f)
{
    float x = __builtin_fmaf(re, kSeqHi, -(float)f);
    x = __builtin_fmaf(re, kSeqLo, x);
    return Comp<float>::apply_sign(__builtin_amdgcn_exp2f(x), im);
}

// ---- waves 0-3: the matrices, one step ahead of the chain, and the outputs
// ADJ: the adjoint recurrence's factors, read from the forward pass's matrices: step s takes the transpose of matrix T - s (any
// matrix for s = 0) and adds left_shift[s] to its log-magnitudes (-inf: a zero matrix).  The matrix is loaded and scaled as it is
// stored, row by row (the same contiguous loads as in the forward pass); the chain reads it by columns, and the shift of a stored
// row j goes with entry j of the vector.
template <bool ADJ, int DEPTH> __device__ __forceinline__ void seq_matrix_waves(const SeqArgs &a, SeqShared &s, int wave, int lane)
{
    static_assert(DEPTH % 2 == 0, "the LDS sets alternate with the step's place in a round");
    typedef Comp<float> C;
    constexpr int D = kSeqD;
    const long long T = a.T;
    const size_t item = blockIdx.x;
    const int row = 8 * wave + (lane >> 3); // eight lanes a row
    const int cq = lane & 7;                // the lane's columns: 4 cq .. 4 cq + 3
    const unsigned char *Ap = a.A + item * (size_t)T * (D * D * 8) + (size_t)(row * D + 4 * cq) * 8;
    [[maybe_unused]] const float *shp = ADJ ? a.left_shift + item * (size_t)T : nullptr;
    const unsigned char *bp = a.bias + item * (size_t)T * (D * 8) + (size_t)row * 8;

    // slot j mod DEPTH: the lane's four entries of the matrix of step j (and, for the adjoint recurrence, the step's shift)
    f4 ra[DEPTH], rb[DEPTH];
    [[maybe_unused]] float qs[DEPTH];
    f2 bq[DEPTH]; // the bias of step j, entry `row`
    constexpr int kNewer = (ADJ ? 4 : 3) * (DEPTH - 1); // loads issued after a slot's own until its turn comes again
    auto load_slot = [&](auto sc, long long j) { // factor of step j (past the end: the last one again)
        constexpr int k = decltype(sc)::value;
        const long long jj = j < T ? j : T - 1;
        if constexpr (ADJ) {
            const long long src = jj > 0 ? T - jj : T - 1;
            load_matrix_part_shift(ra[k], rb[k], bq[k], qs[k], Ap + (size_t)src * (D * D * 8), bp + (size_t)jj * (D * 8), shp + jj);
        } else {
            load_matrix_part(ra[k], rb[k], bq[k], Ap + (size_t)jj * (D * D * 8), bp + (size_t)jj * (D * 8));
        }
    };
    auto wait_slot = [&](auto sc) {
        constexpr int k = decltype(sc)::value;
        if constexpr (ADJ)
            wait_matrix_part_shift<kNewer>(ra[k], rb[k], bq[k], qs[k]);
        else
            wait_matrix_part<kNewer>(ra[k], rb[k], bq[k]);
    };
    static_for<0, DEPTH>([&](auto sc) { load_slot(sc, decltype(sc)::value); });

    // the lane's four entries scaled by the row's power of two and signed, to LDS set `set`
    auto scale_rows = [&](auto sc, int set) {
        constexpr int k = decltype(sc)::value;
        const f4 x = ra[k], y = rb[k];
        float re[4] = {x[0], x[2], y[0], y[2]};
        const float im[4] = {x[1], x[3], y[1], y[3]};
        if constexpr (ADJ) {
#pragma unroll
            for (int e = 0; e < 4; ++e) re[e] += qs[k];
        }
        int key = C::key_of(vmax_raw(vmax_raw(re[0], re[1]), vmax_raw(re[2], re[3])) * kSeqHi);
        key = C::imax(key, C::dpp<0xB1>(key));
        key = C::imax(key, C::dpp<0x4E>(key));
        key = C::imax(key, C::dpp<0x141>(key));
        const float mx = C::of_key(key);
        const bool zero_row = !(mx > -1.0e30f);
        const float nf = zero_row ? 0.0f : __builtin_amdgcn_fmed3f(__builtin_ceilf(mx), -(float)kSeqExpLimit, (float)kSeqExpLimit);
        const float nsub = zero_row ? __builtin_huge_valf() : nf;
        f4 sv;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float xx = __builtin_fmaf(re[e], kSeqHi, -nsub);
            xx = __builtin_fmaf(re[e], kSeqLo, xx);
            const float v = __builtin_amdgcn_exp2f(xx); // 2^-inf = 0 covers zero entries and zero rows
            const float kf = __builtin_fmaf(im[e], 0.318309886183790671538f, 12582912.0f);
            sv[e] = __builtin_bit_cast(float, __builtin_bit_cast(int, v) | (__builtin_bit_cast(int, kf) << 31));
        }
        if constexpr (ADJ) {
            // (rows 33 words apart: the chain's reads by columns then fall on different banks)
#pragma unroll
            for (int e = 0; e < 4; ++e) s.sv[set][row * (D + 1) + 4 * cq + e] = sv[e];
        } else {
            *reinterpret_cast<f4 *>(&s.sv[set][row * D + 4 * cq]) = sv;
        }
        if (cq == 0) {
            // what the chain needs of the row and of its bias, in one 16-byte word
            const f2 b = bq[k];
            const float kf = __builtin_fmaf(b[1], 0.318309886183790671538f, 12582912.0f);
            s.rec[set][row] = int4{(int)nf, exponent_above(b[0]), __builtin_bit_cast(int, b[0]), __builtin_bit_cast(int, kf) << 31};
            if constexpr (ADJ) s.nsrc[set][row] = zero_row ? -kSeqExpLimit : (int)nf; // (a zero row must not set the scale of the vector)
        }
    };

    // the factor of step 0, before the chain's first step
    wait_slot(std::integral_constant<int, 0>{});
    scale_rows(std::integral_constant<int, 0>{}, 0);
    load_slot(std::integral_constant<int, 0>{}, DEPTH);
    lds_barrier();

    // while the chain takes step t: the factor of step t + 1 scaled.  u = t mod DEPTH picks the ring's
    // registers and the LDS sets at compile time
    auto step = [&](auto uc, auto prefetch, [[maybe_unused]] long long t) {
        constexpr int u = decltype(uc)::value;
        constexpr bool kPrefetch = decltype(prefetch)::value; // false after the last full round: the rest of the sequence has landed
        constexpr int slot = (u + 1) % DEPTH;
        if constexpr (kPrefetch) wait_slot(std::integral_constant<int, slot>{});
        scale_rows(std::integral_constant<int, slot>{}, (u + 1) & 1); // (past the end: the last factor again, read by nobody)
        // the registers are free: the factor of step t + 1 + DEPTH (every step of a full round issues its loads)
        if constexpr (kPrefetch) load_slot(std::integral_constant<int, slot>{}, t + 1 + DEPTH);
        lds_barrier();
    };
    long long tb = 0;
    for (; tb + DEPTH <= T; tb += DEPTH) static_for<0, DEPTH>([&](auto uc) { step(uc, std::true_type{}, tb + decltype(uc)::value); });
    // Everything still in flight lands before the last, partial round: from here on the compiler is free to reuse a ring register
    // that no step reads any more, and a load still on its way would overwrite whatever it put there.
    static_for<0, DEPTH>([&](auto sc) { // (every register of the ring passes a wait for all of them)
        constexpr int k = decltype(sc)::value;
        if constexpr (ADJ)
            wait_matrix_part_shift<0>(ra[k], rb[k], bq[k], qs[k]);
        else
            wait_matrix_part<0>(ra[k], rb[k], bq[k]);
    });
    const int rest = (int)(T - tb); // (the same for the whole workgroup)
    static_for<0, DEPTH - 1>([&](auto uc) {
        if (rest > decltype(uc)::value) step(uc, std::false_type{}, tb + decltype(uc)::value);
    });
}

// ---- waves 4-7: the chain
// ADJ: the step's matrix lies in LDS as it is stored, each row j scaled by its own shift n_j, and is applied transposed: entry i of the
// product is the sum over j of (entry (j, i)) (entry j of the vector) 2^(n_j), so n_j joins the exponent of entry j of the vector.
template <bool ADJ> __device__ __forceinline__ void seq_chain_waves(const SeqArgs &a, SeqShared &s, int kw, int lane)
{
    typedef Comp<float> C;
    constexpr int D = kSeqD;
    const long long T = a.T;
    const size_t item = blockIdx.x;
    const int row = 8 * kw + (lane >> 3);
    const int cq = lane & 7;
    const int src_group = cq >> 1; // the group the lane's four entries of the vector belong to
    const float kNegInf = -__builtin_huge_valf();

    // the starting vector goes to the set of LDS words that step 0 reads
    if (kw == 0) {
        const int ent = lane & 31;
        float2 v = float2{kNegInf, 0.0f};
        if (a.h0) v = *reinterpret_cast<const float2 *>(a.h0 + (item * D + ent) * 8);
        int f = exponent_above(v.x);
        f = C::imax(f, C::dpp<0xB1>(f));
        f = C::imax(f, C::dpp<0x4E>(f));
        f = C::imax(f, C::dpp<0x141>(f)); // the eight entries of a group sit in eight adjacent lanes
        s.m[1][ent] = v.x > kNegInf ? scaled_term(v.x, v.y, f) : 0.0f;
        if ((lane & 7) == 0) s.f[1][ent >> 3] = f;
    }
    lds_barrier();

    auto step = [&](auto uc, auto, long long) {
        constexpr int u = decltype(uc)::value;
        constexpr int rs = (u + 1) & 1, ws = u & 1; // sets of the vector read and written (tb is a multiple of the depth, which is even)
        constexpr int ms = u & 1;                   // set of the scaled matrix
        const int4 rec = s.rec[ms][row]; // the row's shift; its bias: exponent, log-magnitude, sign
        const int eb = rec.y;
        const float bre = __builtin_bit_cast(float, rec.z);
        const f4 hm = *reinterpret_cast<const f4 *>(&s.m[rs][4 * cq]);
        const int fsrc = s.f[rs][src_group];
        f4 sv;
        int n, G;
        float part;
        if constexpr (ADJ) {
            // ---- row i of A^T h: the lane's entries j = 4 cq .. 4 cq + 3 of column i, and of the vector with the rows' shifts
#pragma unroll
            for (int e = 0; e < 4; ++e) sv[e] = s.sv[ms][(4 * cq + e) * (D + 1) + row];
            const int4 nj = *reinterpret_cast<const int4 *>(&s.nsrc[ms][4 * cq]);
            const int ej[4] = {nj.x + fsrc, nj.y + fsrc, nj.z + fsrc, nj.w + fsrc};
            int g = C::imax(C::imax(ej[0], ej[1]), C::imax(ej[2], ej[3]));
            g = C::imax(g, C::dpp<0xB1>(g));
            g = C::imax(g, C::dpp<0x4E>(g));
            g = C::imax(g, C::dpp<0x141>(g)); // the row's eight lanes cover all entries of the vector
            G = g;
            n = 0;
            part = 0.0f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int down = ej[e] - G;
                part = __builtin_fmaf(sv[e], __builtin_ldexpf(hm[e], down > -300 ? down : -300), part);
            }
        } else {
            // ---- row i of A_t h_{t-1}: the eight lanes' products on the exponent n_i + G
            sv = *reinterpret_cast<const f4 *>(&s.sv[ms][row * D + 4 * cq]);
            n = rec.x;
            const int4 fa = *reinterpret_cast<const int4 *>(&s.f[rs][0]);
            G = C::imax(C::imax(fa.x, fa.y), C::imax(fa.z, fa.w));
            const int down = fsrc - G;
            part = sv[0] * hm[0];
            part = __builtin_fmaf(sv[1], hm[1], part);
            part = __builtin_fmaf(sv[2], hm[2], part);
            part = __builtin_fmaf(sv[3], hm[3], part);
            part = __builtin_ldexpf(part, down > -300 ? down : -300);
        }
        part = add_dpp<0xB1>(part);
        part = add_dpp<0x4E>(part);
        part = add_dpp<0x141>(part);
        // ---- new exponent of the wave's eight entries: the largest among the eight sums and the eight bias terms
        int ep;
        (void)__builtin_frexpf(part, &ep);
        int F = C::imax(part != 0.0f ? ep + n + G : kSeqNone, eb);
        F = C::imax(F, C::dpp<0x140>(F)); // the other row in these sixteen lanes
        F = C::xor16_imax(F);
        F = C::xor32_imax(F);
        F = F < kSeqNone ? kSeqNone : (F > 2 * kSeqExpLimit ? 2 * kSeqExpLimit : F); // (float log-magnitudes resolve nothing out there)
        const int up = n + G - F; // at most 0 for a non-zero sum
        float mant = __builtin_ldexpf(part, up > -300 ? (up < 300 ? up : 300) : -300);
        float xb = __builtin_fmaf(bre, kSeqHi, -(float)F); // the bias on that exponent (a zero bias, log-magnitude -inf, adds 2^-inf = 0)
        xb = __builtin_fmaf(bre, kSeqLo, xb);
        mant += __builtin_bit_cast(float, __builtin_bit_cast(int, __builtin_amdgcn_exp2f(xb)) | rec.w);
        const bool none = __builtin_amdgcn_ballot_w64(mant != 0.0f) == 0; // a group of zeros carries no exponent
        if (cq == 0) s.m[ws][row] = mant;
        if (lane == 0) s.f[ws][kw] = none ? kSeqNone : F;
        lds_barrier();
    };
    long long tb = 0;
    for (; tb + kSeqDepth <= T; tb += kSeqDepth) {
        step(std::integral_constant<int, 0>{}, std::true_type{}, tb);
        step(std::integral_constant<int, 1>{}, std::true_type{}, tb + 1);
        step(std::integral_constant<int, 2>{}, std::true_type{}, tb + 2);
        step(std::integral_constant<int, 3>{}, std::true_type{}, tb + 3);
        step(std::integral_constant<int, 4>{}, std::true_type{}, tb + 4);
        step(std::integral_constant<int, 5>{}, std::true_type{}, tb + 5);
        step(std::integral_constant<int, 6>{}, std::true_type{}, tb + 6);
        step(std::integral_constant<int, 7>{}, std::true_type{}, tb + 7);
    }
    const int rest = (int)(T - tb);
    if (rest > 0) step(std::integral_constant<int, 0>{}, std::false_type{}, tb);
    if (rest > 1) step(std::integral_constant<int, 1>{}, std::false_type{}, tb + 1);
    if (rest > 2) step(std::integral_constant<int, 2>{}, std::false_type{}, tb + 2);
    if (rest > 3) step(std::integral_constant<int, 3>{}, std::false_type{}, tb + 3);
    if (rest > 4) step(std::integral_constant<int, 4>{}, std::false_type{}, tb + 4);
    if (rest > 5) step(std::integral_constant<int, 5>{}, std::false_type{}, tb + 5);
    if (rest > 6) step(std::integral_constant<int, 6>{}, std::false_type{}, tb + 6);
}

// ---- wave 8: the states out.  While the chain takes step t it reads the state of step t - 1 from LDS and stores it, so that
// neither the chain nor the matrix waves ever wait for a logarithm or a store.
__device__ __forceinline__ void seq_output_wave(const SeqArgs &a, SeqShared &s, int lane)
{
    typedef Comp<float> C;
    constexpr int D = kSeqD;
    const long long T = a.T;
    const size_t item = blockIdx.x;
    const int ent = lane & 31; // the entry this lane handles (the upper half of the wave repeats the lower and stores nothing)
    unsigned char *og = a.out_goom ? a.out_goom + item * (size_t)T * (D * 8) + (size_t)ent * 8 : nullptr;
    float *os = a.out_scaled ? a.out_scaled + item * (size_t)T * D + ent : nullptr;
    float *ol = a.out_logscale ? a.out_logscale + item * (size_t)T : nullptr;
    const float kNegInf = -__builtin_huge_valf();
    // the state held in LDS set `set` (that of step t)
    auto write_state = [&](int set, long long t) {
        const float m = s.m[set][ent];
        const int f = s.f[set][ent >> 3];
        if (og) {
            float2 o;
            o.x = C::out_re_f(m, (float)f); // (-inf for a zero)
            o.y = m < 0.0f ? C::pi() : 0.0f;
            if (lane < D) *reinterpret_cast<float2 *>(og + (size_t)t * (D * 8)) = o;
        }
        if (os || ol) {
            // scaled exponentiation (Section 4.3, eq. 27): with c the log of the largest magnitude, exp(z_i - c + 2) is the entry over the
            // largest entry, times e^2; the exponents only enter c
            const int4 fa = *reinterpret_cast<const int4 *>(&s.f[set][0]);
            const int g = C::imax(C::imax(fa.x, fa.y), C::imax(fa.z, fa.w));
            const int down = f - g;
            const float v = __builtin_ldexpf(m, down > -300 ? down : -300);
            float am = __builtin_fabsf(v);
            am = C::group_allmax<32>(am, am);
            if (os && lane < D) os[(size_t)t * D] = am > 0.0f ? v * (7.38905609893065022723f * __builtin_amdgcn_rcpf(am)) : 0.0f;
            if (ol && lane == 0) ol[t] = am > 0.0f ? (float)(((double)C::log2_abs(am) + (double)g) * 0.693147180559945309417) : kNegInf;
        }
    };

    lds_barrier(); // the set-up of the other waves
    for (long long t = 0; t < T; ++t) {
        if (t > 0) write_state((int)((t + 1) & 1), t - 1);
        lds_barrier();
    }
    write_state((int)((T - 1) & 1), T - 1);
}

// All three kinds of waves pass the same barriers: one after their set-up, one at the end of every step.
template <bool ADJ> __global__ __launch_bounds__(kSeqThreads) void affine_seq_kernel(SeqArgs a)
{
    __shared__ __align__(16) SeqShared s;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (wave < 4)
        seq_matrix_waves<ADJ, ADJ ? kSeqRingAdj : kSeqRing>(a, s, wave, lane);
    else if (wave < 8)
        seq_chain_waves<ADJ>(a, s, wave - 4, lane);
    else
        seq_output_wave(a, s, lane);
}

} // namespace

// every sequence of the batch by one workgroup, start to end; the caller has checked pointers and sizes
int launch_affine_seq(goom_ctx *ctx, const void *A, const void *bias, const void *h0, void *H, void *scaled, void *logscale, long long T, long long batch,
                      const float *adjoint_shift)
{
    if (T <= 0 || batch <= 0) return GOOM_OK;
    if (batch > 0x7fffffffLL) return goom::fail(ctx, GOOM_EUNSUPPORTED, "too many sequences for one launch (%lld)", batch);
    SeqArgs args;
    args.A = static_cast<const unsigned char *>(A);
    args.bias = static_cast<const unsigned char *>(bias);
    args.h0 = static_cast<const unsigned char *>(h0);
    args.out_goom = static_cast<unsigned char *>(H);
    args.out_scaled = static_cast<float *>(scaled);
    args.out_logscale = static_cast<float *>(logscale);
    args.left_shift = adjoint_shift;
    args.T = T;
    goom::prof_begin(ctx, "affine_sequential_walk");
    if (adjoint_shift)
        hipLaunchKernelGGL(affine_seq_kernel<true>, dim3((unsigned)batch), dim3(kSeqThreads), 0, ctx->stream, args);
    else
        hipLaunchKernelGGL(affine_seq_kernel<false>, dim3((unsigned)batch), dim3(kSeqThreads), 0, ctx->stream, args);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch affine_seq_kernel");
}

} // namespace goom_chain
