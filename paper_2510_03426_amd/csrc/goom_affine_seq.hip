// Linear recurrence with bias, h_t = A_t h_{t-1} + b_t over GOOMs (paper Section 4.3), float components, d = 32, for
// batches of many sequences: one workgroup walks one whole sequence, step after step, and reads every matrix once.
//
// With a hundred sequences or more there is no need to cut a sequence into chunks (whose products cost a matrix-matrix
// product per step and a second pass over the matrices): a workgroup of eight waves keeps eight steps of its sequence's
// matrices in flight, which is enough outstanding memory traffic per compute unit, and a step is a matrix-vector product
// spread over the 512 lanes:
//
//   * a lane loads two adjacent entries of a row (16 bytes; the workgroup's loads of a step cover the 8 KiB matrix
//     contiguously), the sixteen lanes of a row agree on the row's power-of-two shift n_i and scale their entries to
//     (+-) 2^(log2|A_ij| - n_i);
//   * the vector lives in LDS as float mantissas with one whole-number exponent per group of four entries (the four rows
//     a wave produces); a lane reads its two entries, brings them to the largest group exponent G and the row's sixteen
//     lanes add up their products: entry i of A_t h is that sum times 2^(n_i + G);
//   * the bias b_i joins on the new exponent of the wave's four rows (the largest of the four sums' and the four bias
//     terms' exponents), the wave writes four mantissas and that exponent, and one workgroup barrier ends the step
//     (mantissas and exponents alternate between two sets of LDS words, so one barrier a step is enough).
//
// The state of step t - 1 leaves during step t, through one wave (the waves take turns): as a GOOM, and / or as the
// scaled exponential of Section 4.3, eq. 27 with its log-scaling constant.  Nothing but A_t, b_t (read once) and the
// outputs (written once) touches HBM.
#include "goom_chain_fast.h"
#include <type_traits>

namespace goom_chain {

namespace {

constexpr int kSeqDepth = 8;          // steps of a sequence in flight, per lane one 16-byte piece of each
constexpr int kSeqNone = -(1 << 28);  // exponent of a group of zeros
constexpr int kSeqExpLimit = 1 << 27; // whole-number exponents are kept inside +- this

struct SeqArgs {
    const unsigned char *A;    // [batch, T, 32, 32] complex64
    const unsigned char *bias; // [batch, T, 32] complex64
    const unsigned char *h0;   // NULL (zero) or [batch, 32] complex64
    unsigned char *out_goom;   // NULL or [batch, T, 32] complex64
    float *out_scaled;         // NULL or [batch, T, 32]
    float *out_logscale;       // NULL or [batch, T]
    long long T;
};

// Workgroup barrier that orders LDS traffic only: the matrices in flight from HBM stay in flight across it (the
// general barrier would wait for every outstanding load, and with it for the whole ring of prefetched steps).
__device__ inline void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// The ring of prefetched steps: loads the compiler does not track (it would make every step wait for the loads issued in it,
// to copy what they fetched to the registers of the step that consumes it), issued and awaited by hand.  A load's registers
// pass through wait_ring before their first use, so nothing reads them earlier; vector-memory loads return in the order of
// issue, and stores issued in between only make the wait stricter.
typedef float f2 __attribute__((ext_vector_type(2)));
__device__ inline void load_ring(f4 &m, f2 &b, const unsigned char *pm, const unsigned char *pb)
{
    asm volatile("global_load_dwordx4 %0, %2, off\n\tglobal_load_dwordx2 %1, %3, off" : "=&v"(m), "=&v"(b) : "v"(pm), "v"(pb) : "memory");
}
// the pair issued kSeqDepth steps ago has landed once at most 2 (kSeqDepth - 1) newer loads are outstanding
template <int NEWER> __device__ inline void wait_ring(f4 &m, f2 &b)
{
    asm volatile("s_waitcnt vmcnt(%2)" : "+v"(m), "+v"(b) : "n"(NEWER) : "memory");
}

__device__ inline int imax3(int a, int b, int c)
{
    const int m = a > b ? a : b;
    return m > c ? m : c;
}

__global__ __launch_bounds__(512) void affine_seq_kernel(SeqArgs a)
{
    typedef Comp<float> C;
    constexpr int D = 32;
    __shared__ __align__(16) float mbuf[2][D];   // mantissas of the vector
    __shared__ __align__(16) int fbuf[2][D / 4]; // exponent of entries 4 w .. 4 w + 3 (the rows wave w produces)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int row = tid >> 4;         // sixteen lanes a row
    const int cpos = tid & 15;        // the lane's columns: 2 cpos, 2 cpos + 1
    const int src_group = cpos >> 1;  // the group those two entries of the vector belong to
    const int ent = lane & 31;        // entry handled when this wave writes a state out
    const long long T = a.T;
    const size_t item = blockIdx.x;
    const unsigned char *Ap = a.A + item * (size_t)T * (D * D * 8) + (size_t)tid * 16;
    const unsigned char *bp = a.bias + item * (size_t)T * (D * 8) + (size_t)row * 8;
    unsigned char *og = a.out_goom ? a.out_goom + item * (size_t)T * (D * 8) + (size_t)ent * 8 : nullptr;
    float *os = a.out_scaled ? a.out_scaled + item * (size_t)T * D + ent : nullptr;
    float *ol = a.out_logscale ? a.out_logscale + item * (size_t)T : nullptr;
    const float kHi = 1.44269502162933349609375f; // float nearest log2(e)
    const float kLo = 1.925963033500011e-8f;      // log2(e) - kHi
    const float kNegInf = -__builtin_huge_valf();

    // whole-number exponent at or above log2 of a magnitude given by its natural logarithm; kSeqNone for a zero
    auto exponent_above = [&](float re) {
        const float e = __builtin_amdgcn_fmed3f(__builtin_ceilf(re * kHi), -(float)kSeqExpLimit, (float)kSeqExpLimit);
        return re > kNegInf ? (int)e : kSeqNone;
    };
    // (+-) 2^(re log2(e) - f) for a whole number f, the product with log2(e) carried in two floats
    auto scaled_term = [&](float re, float im, int f) {
        float x = __builtin_fmaf(re, kHi, -(float)f);
        x = __builtin_fmaf(re, kLo, x);
        return C::apply_sign(__builtin_amdgcn_exp2f(x), im);
    };

    // the starting vector goes to the set of LDS words that step 0 reads
    if (wave == 0) {
        float2 v = float2{kNegInf, 0.0f};
        if (a.h0) v = *reinterpret_cast<const float2 *>(a.h0 + (item * D + ent) * 8);
        int f = exponent_above(v.x);
        f = C::imax(f, C::dpp<0xB1>(f));
        f = C::imax(f, C::dpp<0x4E>(f)); // the four entries of a group sit in one quad of lanes
        mbuf[1][ent] = v.x > kNegInf ? scaled_term(v.x, v.y, f) : 0.0f;
        if ((lane & 3) == 0) fbuf[1][ent >> 2] = f;
    }

    f4 ring[kSeqDepth];
    f2 bring[kSeqDepth];
#pragma unroll
    for (int u = 0; u < kSeqDepth; ++u) {
        const long long t = u < T ? u : T - 1;
        load_ring(ring[u], bring[u], Ap + (size_t)t * (D * D * 8), bp + (size_t)t * (D * 8));
    }
    __syncthreads();

    // the state held in LDS set `set` (that of step t) leaves through this wave's lanes
    auto write_state = [&](int set, long long t) {
        const float m = mbuf[set][ent];
        const int f = fbuf[set][ent >> 2];
        if (og) {
            float2 o;
            o.x = C::out_re_f(m, (float)f); // (-inf for a zero)
            o.y = m < 0.0f ? C::pi() : 0.0f;
            if (lane < D) *reinterpret_cast<float2 *>(og + (size_t)t * (D * 8)) = o;
        }
        if (os || ol) {
            // scaled exponentiation (Section 4.3, eq. 27): with c the log of the largest magnitude, exp(z_i - c + 2) is the entry over the
            // largest entry, times e^2; the exponents only enter c
            int g = f;
            g = C::imax(g, C::dpp<0x141>(g));
            g = C::imax(g, C::dpp<0x140>(g)); // over the four groups of a row of sixteen lanes
            g = C::xor16_imax(g);             // all eight groups
            const int down = f - g;
            const float v = __builtin_ldexpf(m, down > -300 ? down : -300);
            float am = __builtin_fabsf(v);
            am = C::group_allmax<32>(am, am);
            if (os && lane < D) os[(size_t)t * D] = am > 0.0f ? v * (7.38905609893065022723f / am) : 0.0f;
            if (ol && lane == 0) ol[t] = am > 0.0f ? (float)(((double)C::log2_abs(am) + (double)g) * 0.693147180559945309417) : kNegInf;
        }
    };

    // one step; u = t mod kSeqDepth picks the ring's registers and the LDS sets at compile time
    auto step = [&](auto uc, auto prefetch, long long t) {
        constexpr int u = decltype(uc)::value;
        constexpr bool kPrefetch = decltype(prefetch)::value; // false after the last full round: the rest of the sequence has landed
        constexpr int kOdd = 1; // (tb is a multiple of the depth, which is even: the sets alternate with u)
        const int rs = (u + kOdd) & 1, ws = u & 1;
        // ---- the vector of step t - 1
        const float2 mm = *reinterpret_cast<const float2 *>(&mbuf[rs][2 * cpos]);
        const int fsrc = fbuf[rs][src_group];
        const int4 fa = *reinterpret_cast<const int4 *>(&fbuf[rs][0]);
        const int4 fb = *reinterpret_cast<const int4 *>(&fbuf[rs][4]);
        if (t > 0 && wave == u) write_state(rs, t - 1);
        // ---- this step's matrix: the row's shift, the lane's two entries scaled and signed
        if constexpr (kPrefetch) wait_ring<2 * (kSeqDepth - 1)>(ring[u], bring[u]);
        const f4 raw = ring[u];
        const f2 b = bring[u];
        int key = C::key_of(vmax_raw(raw[0], raw[2]) * kHi);
        key = C::imax(key, C::dpp<0xB1>(key));
        key = C::imax(key, C::dpp<0x4E>(key));
        key = C::imax(key, C::dpp<0x141>(key));
        key = C::imax(key, C::dpp<0x140>(key));
        const float mx = C::of_key(key);
        const bool zero_row = !(mx > -1.0e30f);
        const float nf = zero_row ? 0.0f : __builtin_amdgcn_fmed3f(__builtin_ceilf(mx), -(float)kSeqExpLimit, (float)kSeqExpLimit);
        const float nsub = zero_row ? __builtin_huge_valf() : nf;
        const int n = (int)nf;
        float sv[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            float x = __builtin_fmaf(raw[2 * e], kHi, -nsub);
            x = __builtin_fmaf(raw[2 * e], kLo, x);
            const float v = __builtin_amdgcn_exp2f(x); // 2^-inf = 0 covers zero entries and zero rows
            const float kf = __builtin_fmaf(raw[2 * e + 1], 0.318309886183790671538f, 12582912.0f);
            sv[e] = __builtin_bit_cast(float, __builtin_bit_cast(int, v) | (__builtin_bit_cast(int, kf) << 31));
        }
        const int eb = exponent_above(b[0]);
        // ---- row i of A_t h_{t-1}: the sixteen lanes' products on the exponent n_i + G
        const int G = imax3(imax3(fa.x, fa.y, fa.z), imax3(fa.w, fb.x, fb.y), C::imax(fb.z, fb.w));
        const int down = fsrc - G;
        float part = __builtin_fmaf(sv[0], mm.x, sv[1] * mm.y);
        part = __builtin_ldexpf(part, down > -300 ? down : -300);
        part = add_dpp<0xB1>(part);
        part = add_dpp<0x4E>(part);
        part = add_dpp<0x141>(part);
        part = add_dpp<0x140>(part);
        // ---- new exponent of the wave's four entries: the largest among the four sums and the four bias terms
        int ep;
        (void)__builtin_frexpf(part, &ep);
        const int erow = C::imax(part != 0.0f ? ep + n + G : kSeqNone, eb);
        int F = C::xor16_imax(erow);
        F = C::xor32_imax(F);
        F = F > kSeqNone ? (F < 2 * kSeqExpLimit ? F : 2 * kSeqExpLimit) : kSeqNone; // (float log-magnitudes resolve nothing out there)
        const int up = n + G - F; // at most 0 for a non-zero sum
        float mant = __builtin_ldexpf(part, up > -300 ? (up < 300 ? up : 300) : -300);
        mant += scaled_term(b[0], b[1], F); // (a zero bias, log-magnitude -inf, adds 2^-inf = 0)
        const bool none = __builtin_amdgcn_ballot_w64(mant != 0.0f) == 0; // a group of zeros carries no exponent
        if (cpos == 0) mbuf[ws][row] = mant;
        if (lane == 0) fbuf[ws][wave] = none ? kSeqNone : F;
        if constexpr (kPrefetch) {
            // the registers are free: step t + kSeqDepth (past the end the last step again: every step of a full round issues its pair)
            const long long tn = t + kSeqDepth < T ? t + kSeqDepth : T - 1;
            load_ring(ring[u], bring[u], Ap + (size_t)tn * (D * D * 8), bp + (size_t)tn * (D * 8));
        }
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
    static_assert(kSeqDepth == 8, "the steps are written out");
    // Everything still in flight lands before the last, partial round: from here on the compiler is free to reuse a ring register
    // that no step reads any more, and a load still on its way would overwrite whatever it put there.
    asm volatile("s_waitcnt vmcnt(0)"
                 : "+v"(ring[0]), "+v"(ring[1]), "+v"(ring[2]), "+v"(ring[3]), "+v"(ring[4]), "+v"(ring[5]), "+v"(ring[6]), "+v"(ring[7]), "+v"(bring[0]),
                   "+v"(bring[1]), "+v"(bring[2]), "+v"(bring[3]), "+v"(bring[4]), "+v"(bring[5]), "+v"(bring[6]), "+v"(bring[7])
                 :
                 : "memory");
    const int rest = (int)(T - tb); // (the same for the whole workgroup)
    if (rest > 0) step(std::integral_constant<int, 0>{}, std::false_type{}, tb);
    if (rest > 1) step(std::integral_constant<int, 1>{}, std::false_type{}, tb + 1);
    if (rest > 2) step(std::integral_constant<int, 2>{}, std::false_type{}, tb + 2);
    if (rest > 3) step(std::integral_constant<int, 3>{}, std::false_type{}, tb + 3);
    if (rest > 4) step(std::integral_constant<int, 4>{}, std::false_type{}, tb + 4);
    if (rest > 5) step(std::integral_constant<int, 5>{}, std::false_type{}, tb + 5);
    if (rest > 6) step(std::integral_constant<int, 6>{}, std::false_type{}, tb + 6);
    if (wave == 0) write_state((int)((T - 1) & 1), T - 1);
}

} // namespace

// every sequence of the batch by one workgroup, start to end; the caller has checked pointers and sizes
int launch_affine_seq(goom_ctx *ctx, const void *A, const void *bias, const void *h0, void *H, void *scaled, void *logscale, long long T, long long batch)
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
    args.T = T;
    goom::prof_begin(ctx, "affine_sequential_walk");
    hipLaunchKernelGGL(affine_seq_kernel, dim3((unsigned)batch), dim3(512), 0, ctx->stream, args);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch affine_seq_kernel");
}

} // namespace goom_chain
