// Repair pass of LMME (paper Section 3.2): recompute, by the definition
//     C'_ik = LSE_j(A'_ij + B'_jk)                                   (Section 3.2, eq. 9: the definition)
// every output whose scaled real product (eq. 10, computed by the chain kernel) may have lost
// terms to underflow.  The paper itself calls the scaled product a compromise in precision;
// when the logarithms of the operands spread over hundreds of units, almost every term sits
// below the component format's range after the row/column shifts and the product comes out
// as zero although the true value is finite.
//
// Certificate.  With row shifts n_i and column shifts e_k (whole powers of two, largest entry
// of the row / column scaled to at most 1), a term that is dropped is smaller than the
// smallest normal number 2^-E of the format, so the dropped mass of one output is below
// d 2^-E.  An output whose scaled magnitude log2|C~_ik| = Re(C'_ik) log2(e) - n_i - e_k is
// at least -E + log2(d) + 20 is therefore right to about 2^-20 relative and is kept; all
// others are recomputed term by term on the vector ALUs, in two passes over j (maximum, then
// signed sum of exponentials), which never leaves the representable range.
//
// Outputs are handled in blocks of 64 x 64 of one batch item, a thread 4 x 4 of them, so that
// one pair of LDS reads serves sixteen terms; the rows of A and the columns of B are staged in LDS 32
// inner indices at a time.  The certificate only needs the row maxima of A' and the column maxima of B'
// (one light pass over the operands, made once by a workgroup for the 128 x 128 outputs = four blocks that
// it owns, so that the operands of a 128 x 128 x 128 product are read once): a block whose outputs are all
// certified ends there; one
// with few outputs to repair hands them to its waves one at a time; only a block with many (float
// components on wide-range data) runs the two sweeps over all sixteen positions per thread, or, with float
// components and at most 128 inner indices, orders the terms of every output first and finishes most outputs from
// their one or two leading terms.
#include <type_traits>

#include "goom_chain_kernel.h"

namespace {

constexpr int kTile = 16;
constexpr int kThreads = kTile * kTile;

struct ExactArgs {
    const void *A, *B;
    const void *shifts; // NULL, or the product kernel's row and column shifts ([batch][2][128], n = m = 128 only)
    void *C;
    long long batch;
    int n, d, m;
    float pos_inf; // +infinity
};

template <typename R> struct Num;
template <> struct Num<float> {
    static constexpr float kLog2e = 1.44269504088896340736f;
    static constexpr float kLn2 = 0.693147180559945309417f;
    static constexpr float kMargin = -126.0f + 20.0f;
    __device__ static float neg_inf() { return -__builtin_huge_valf(); }
    __device__ static float pi() { return 3.14159274101257324219f; }
    __device__ static float exp2_(float x) { return __builtin_amdgcn_exp2f(x); }
    __device__ static float max_(float x, float y) { return __builtin_fmaxf(x, y); }
    __device__ static float fma_(float x, float y, float z) { return __builtin_fmaf(x, y, z); }
    __device__ static float log2_(float x) { return ::log2f(x); }
    __device__ static int parity(float im) { return (int)__builtin_rintf(im * 0.318309886183790671538f) & 1; }
};
template <> struct Num<double> {
    static constexpr double kLog2e = 1.44269504088896340736;
    static constexpr double kLn2 = 0.693147180559945309417;
    static constexpr double kMargin = -1022.0 + 40.0;
    __device__ static double neg_inf() { return -__builtin_huge_val(); }
    __device__ static double pi() { return 3.14159265358979311600; }
    __device__ static double max_(double x, double y) { return __builtin_fmax(x, y); }
    __device__ static double fma_(double x, double y, double z) { return __builtin_fma(x, y, z); }
    __device__ static double exp2_(double x) // x <= 0: whole part split off, short series for the rest
    {
        const double k = __builtin_rint(x);
        const double y = __builtin_ldexp(goom_chain::Comp<double>::exp2_small(x - k), (int)(k > -4000.0 ? k : -4000.0));
        return x > -1200.0 ? y : 0.0;
    }
    __device__ static double log2_(double x) { return ::log2(x); }
    __device__ static int parity(double im) { return (int)__builtin_rint(im * 0.318309886183790671538) & 1; }
};

constexpr int kOut = 64;    // outputs are worked off in blocks of 64 x 64, a thread 4 x 4 of them
// Outputs a workgroup owns, kSuper x kSuper.  Double components: 128 (four blocks), the maxima taken once for all
// of them; repairs are rare there and the pass over the operands is what the kernel costs (config 3: 2.7 -> 2.2 ms).
// Float components on wide-range data spend their time in the sweeps, and one block per workgroup is faster
// (4.45 against 4.8 ms).
template <typename R> constexpr int super_block() { return sizeof(R) == 8 ? 128 : 64; }
constexpr int kJBlock = 32; // inner indices staged in LDS at a time
constexpr int kMaxList = 256; // a block with at most this many outputs to repair handles them one by one

template <typename R> __device__ inline R flip_sign(R x, float signword);
template <> __device__ inline float flip_sign<float>(float x, float signword)
{
    return __builtin_bit_cast(float, __builtin_bit_cast(unsigned, x) ^ __builtin_bit_cast(unsigned, signword));
}
template <> __device__ inline double flip_sign<double>(double x, float signword)
{
    return __builtin_bit_cast(double, __builtin_bit_cast(unsigned long long, x) ^ ((unsigned long long)__builtin_bit_cast(unsigned, signword) << 32));
}

// KEYED (float components, at most 128 inner indices): a block with many outputs to repair orders the terms of
// each by keys first and finishes most outputs from their one or two leading terms (see below); it then holds
// all of its operands in LDS, which leaves room for two workgroups on a compute unit.
constexpr int kKeyedMaxInner = 128;
constexpr int kKeyedLda = kKeyedMaxInner + 1;
constexpr size_t kKeyedLds = (size_t)kOut * kKeyedLda * 4 + (size_t)kKeyedMaxInner * kOut * 4 + 2 * kThreads * 4 + kOut * kOut * 2;

template <typename R, bool KEYED> __global__ __launch_bounds__(kThreads, sizeof(R) == 4 && !KEYED ? 4 : 2) void lmme_exact_kernel(ExactArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int n = a.n, d = a.d, m = a.m;
    constexpr int kSuper = super_block<R>();
    constexpr int LDA = kJBlock + 1; // rows of A: [i][j], padded so that the four rows a wave reads at once differ in bank
    // LDS: log-magnitudes of 64 rows of A [64][33] and 64 columns of B [32][64]; their signs as float +-0
    R *are = reinterpret_cast<R *>(smem);
    R *bre = are + kOut * LDA;
    float *asg = reinterpret_cast<float *>(bre + kJBlock * kOut);
    float *bsg = asg + kOut * LDA;

    const int tid = threadIdx.x;
    const int ty = tid / 16, tx = tid % 16;
    // a workgroup owns kSuper x kSuper outputs of one batch item: the maxima are taken once for all of them, then its
    // (up to) four kOut x kOut blocks are worked off one after the other
    const int blocks_k = (m + kSuper - 1) / kSuper, blocks_i = (n + kSuper - 1) / kSuper;
    // Workgroups go to the eight XCDs in turn, each with an L2 of its own: renumber them so that the blocks of
    // one batch item (which share rows of A' and columns of B') run on the same XCD, one after the other.
    unsigned bid = blockIdx.x; // (the launcher keeps the grid below 2^31)
    const unsigned per_item = (unsigned)blocks_i * (unsigned)blocks_k;
    {
        const unsigned long long span = 8ull * per_item;
        if (span <= gridDim.x) {
            const unsigned sp = (unsigned)span;
            if (bid < gridDim.x / sp * sp) {
                const unsigned grp = bid / sp, r = bid % sp;
                bid = (grp * 8 + r % 8) * per_item + r / 8;
            }
        }
    }
    const long long b = bid / per_item;
    const int rem = (int)(bid % per_item);
    const int I0 = (rem / blocks_k) * kSuper, K0 = (rem % blocks_k) * kSuper;
    int i0 = I0, k0 = K0; // the block in hand
    const R *Ab = static_cast<const R *>(a.A) + (size_t)b * n * d * 2;
    const R *Bb = static_cast<const R *>(a.B) + (size_t)b * d * m * 2;
    R *Cb = static_cast<R *>(a.C) + (size_t)b * n * m * 2;

    // stage inner indices [j0, j0 + 32) of the 64 rows of A and the 64 columns of B (zeros past the edges)
    auto stage = [&](int j0) {
        __syncthreads();
        for (int e = tid; e < kOut * kJBlock; e += kThreads) {
            const int r = e / kJBlock, j = e % kJBlock; // consecutive threads walk along a row of A
            const bool ok = i0 + r < n && j0 + j < d;
            R re = Num<R>::neg_inf();
            float sg = 1.0f; // A's sign as +-1, B's as a sign word: one xor gives the factor of a term
            if (ok) {
                const R *p = Ab + ((size_t)(i0 + r) * d + j0 + j) * 2;
                re = p[0];
                sg = Num<R>::parity(p[1]) ? -1.0f : 1.0f;
            }
            are[r * LDA + j] = re;
            asg[r * LDA + j] = sg;
        }
        for (int e = tid; e < kJBlock * kOut; e += kThreads) {
            const int j = e / kOut, c = e % kOut; // consecutive threads walk along a row of B
            const bool ok = k0 + c < m && j0 + j < d;
            R re = Num<R>::neg_inf();
            float sg = 0.0f;
            if (ok) {
                const R *p = Bb + ((size_t)(j0 + j) * m + k0 + c) * 2;
                re = p[0];
                sg = Num<R>::parity(p[1]) ? -0.0f : 0.0f;
            }
            bre[j * kOut + c] = re;
            bsg[j * kOut + c] = sg;
        }
        __syncthreads();
    };

    // ---- row maxima of A' and column maxima of B' over the whole inner index: all the certificate needs.
    // Straight from memory: a wave takes sixteen rows of A' (its lanes along the row, then a reduction across
    // the lanes) and a quarter of the inner indices of B' (its lanes along the 64 columns).
    __shared__ R s_amax[kSuper], s_bmax[kSuper], s_part[kThreads / 64][kOut];
    __shared__ int s_count;
    __shared__ int s_list[kMaxList];
    const bool given = a.shifts != nullptr; // the shifts come from the product kernel: no pass over the operands
    if (given) {
        const R *sh = static_cast<const R *>(a.shifts) + (size_t)b * 256;
        for (int t = tid; t < kSuper; t += kThreads) {
            s_amax[t] = sh[I0 + t];
            s_bmax[t] = sh[128 + K0 + t];
        }
        __syncthreads();
    }
#pragma unroll 1
    for (int h = 0; h < (given ? 0 : kSuper / kOut); ++h) {
        i0 = I0 + h * kOut;
        k0 = K0 + h * kOut;
        const int lane = tid & 63, wave = tid >> 6;
        R v[16];
#pragma unroll
        for (int rr = 0; rr < 16; ++rr) v[rr] = Num<R>::neg_inf();
        for (int j = lane; j < d; j += 64) {
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) {
                const int i = i0 + 16 * wave + rr;
                if (i < n) v[rr] = Num<R>::max_(v[rr], Ab[((size_t)i * d + j) * 2]);
            }
        }
#pragma unroll
        for (int rr = 0; rr < 16; ++rr) {
            R w = v[rr];
#pragma unroll
            for (int sft = 1; sft < 64; sft <<= 1) w = Num<R>::max_(w, (R)__shfl_xor(w, sft, 64));
            if (lane == 0) s_amax[h * kOut + 16 * wave + rr] = w;
        }
        R cmaxv = Num<R>::neg_inf();
        const int k = k0 + lane;
        if (k < m) {
            R part[4] = {Num<R>::neg_inf(), Num<R>::neg_inf(), Num<R>::neg_inf(), Num<R>::neg_inf()};
            int j = wave;
            for (; j + 12 < d; j += 16) {
#pragma unroll
                for (int u = 0; u < 4; ++u) part[u] = Num<R>::max_(part[u], Bb[((size_t)(j + 4 * u) * m + k) * 2]);
            }
            for (; j < d; j += 4) part[0] = Num<R>::max_(part[0], Bb[((size_t)j * m + k) * 2]);
            cmaxv = Num<R>::max_(Num<R>::max_(part[0], part[1]), Num<R>::max_(part[2], part[3]));
        }
        s_part[wave][lane] = cmaxv;
        __syncthreads();
        if (tid < kOut) {
            R w = s_part[0][tid];
#pragma unroll
            for (int u = 1; u < kThreads / 64; ++u) w = Num<R>::max_(w, s_part[u][tid]);
            s_bmax[h * kOut + tid] = w;
        }
        __syncthreads();
    }

    // ---- one kOut x kOut block: certificate, then the repairs
    auto repair_block = [&](const R *blk_amax, const R *blk_bmax) __attribute__((always_inline)) {
    R amax[4], bmax[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        amax[r] = blk_amax[4 * ty + r];
        bmax[r] = blk_bmax[4 * tx + r];
    }
    // ---- certificate: which outputs of the scaled product may have lost terms to underflow
    unsigned need = 0;
    R log2d = 0;
    for (int s = 1; s < d; s <<= 1) log2d += 1;
    R cre[4][4]; // (all sixteen loads first, from addresses held inside the output, so that they are in flight together)
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int i = i0 + 4 * ty + r, k = k0 + 4 * tx + c;
            if constexpr (KEYED) // (offsets of 32 bits: the launcher checks)
                cre[r][c] = Cb[((unsigned)(i < n ? i : n - 1) * (unsigned)m + (unsigned)(k < m ? k : m - 1)) * 2u];
            else
                cre[r][c] = Cb[((size_t)(i < n ? i : n - 1) * m + (k < m ? k : m - 1)) * 2];
        }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int i = i0 + 4 * ty + r, k = k0 + 4 * tx + c;
            // (given shifts are whole numbers already, with -1e30 for a row or column without a finite entry)
            const R none = given ? (R)-1.0e29 : Num<R>::neg_inf();
            if (i < n && k < m && amax[r] > none && bmax[c] > none) {
                const R ni = given ? amax[r] : (R)__builtin_ceil((double)amax[r] * 1.44269504088896340736);
                const R ek = given ? bmax[c] : (R)__builtin_ceil((double)bmax[c] * 1.44269504088896340736);
                const R scaled = cre[r][c] * Num<R>::kLog2e - ni - ek; // log2 of the scaled product's magnitude
                if (!(scaled >= Num<R>::kMargin + log2d + 1)) need |= 1u << (4 * r + c); // also for -inf and NaN
            }
            // a zero row or column gives an exact zero either way
        }
    // the block's outputs to repair, as a list: a short one is worked off output by output
    __syncthreads(); // (the block before this one is done with the list)
    if (tid == 0) s_count = 0;
    __syncthreads();
    {   // (a wave reserves room for all of its lanes' outputs at once: one atomic a wave)
        const int lane = tid & 63, mine = __builtin_popcount(need);
        int before = mine; // inclusive prefix sum over the wave
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            const int o = __shfl_up(before, s, 64);
            if (lane >= s) before += o;
        }
        int first = 0;
        if (lane == 63 && before > 0) first = atomicAdd(&s_count, before);
        first = __shfl(first, 63, 64);
        int slot = first + before - mine;
        for (unsigned rest = need; rest != 0 && slot < kMaxList; rest &= rest - 1, ++slot) {
            const int q = __builtin_ctz(rest);
            s_list[slot] = (4 * ty + q / 4) * kOut + 4 * tx + q % 4;
        }
    }
    __syncthreads();
    const int count = s_count;
    if (count == 0) return;
    if (count <= kMaxList) {
        // ---- few outputs (the usual case with double components): one wave per output, its lanes
        // share the inner index; operands come straight from memory (they were read a moment ago)
        const int lane = tid & 63, wave = tid >> 6;
        for (int e = wave; e < count; e += kThreads / 64) {
            const int i = i0 + s_list[e] / kOut, k = k0 + s_list[e] % kOut;
            R zmax = Num<R>::neg_inf();
            for (int j = lane; j < d; j += 64)
                zmax = Num<R>::max_(zmax, Ab[((size_t)i * d + j) * 2] + Bb[((size_t)j * m + k) * 2]);
            for (int s = 1; s < 64; s <<= 1) zmax = Num<R>::max_(zmax, __shfl_xor(zmax, s, 64));
            R sv = 0;
            if (zmax > Num<R>::neg_inf()) {
                for (int j = lane; j < d; j += 64) {
                    const R *pa = Ab + ((size_t)i * d + j) * 2, *pb = Bb + ((size_t)j * m + k) * 2;
                    const R t = Num<R>::exp2_(((pa[0] + pb[0]) - zmax) * Num<R>::kLog2e);
                    sv += ((Num<R>::parity(pa[1]) ^ Num<R>::parity(pb[1])) & 1) ? -t : t;
                }
                for (int s = 1; s < 64; s <<= 1) sv += __shfl_xor(sv, s, 64);
            }
            if (lane == 0) {
                R re_out = Num<R>::neg_inf(), im_out = 0;
                if (zmax > Num<R>::neg_inf() && sv != 0) {
                    re_out = zmax + Num<R>::log2_(sv < 0 ? -sv : sv) * Num<R>::kLn2;
                    im_out = sv < 0 ? Num<R>::pi() : (R)0;
                }
                Cb[((size_t)i * m + k) * 2] = re_out;
                Cb[((size_t)i * m + k) * 2 + 1] = im_out;
            }
        }
        return;
    }

    if constexpr (KEYED) {
        // ---- many outputs to repair, float components on wide-range data: one or two terms decide most outputs,
        // and the exponentials of all the others are work for nothing.  A first sweep orders the terms: every
        // log-magnitude as a whole number of 1/16 units below the block's largest (at most 4096 units below: what
        // is smaller counts as that, so a key never understates a term by more than the rounding), plus, for B',
        // the inner index over 128 as a fraction.  Sums of such numbers are exact in float, so one addition gives
        // a term's key, index included, and three more instructions keep the three largest keys of an output.  The
        // operands themselves wait in registers meanwhile and then take the keys' place in LDS; the two leading
        // terms are read back by index, and an output is finished from them when all other terms together,
        // bounded through the third key, cannot move the result's last place.  What is left (about two per cent
        // at N(0, 200^2)) is summed in full, an output to a lane.
        constexpr int kHeld = kOut * kKeyedMaxInner / kThreads; // 32 entries of each operand to a thread
        float *kx = reinterpret_cast<float *>(smem), *ky = kx + kOut * kKeyedLda; // keys, then the operands: [64][129], [128][64]
        unsigned *sa = reinterpret_cast<unsigned *>(ky + kKeyedMaxInner * kOut), *sb = sa + kThreads; // signs, a word to a thread
        unsigned short *open = reinterpret_cast<unsigned short *>(sb + kThreads);
        float ablk = Num<float>::neg_inf(), bblk = Num<float>::neg_inf(); // upper bounds of the block's operands
        {
            const int lane = tid & 63;
            const float av = blk_amax[lane], bv = blk_bmax[lane];
            ablk = given ? (av > -1.0e29f ? av * Num<float>::kLn2 : Num<float>::neg_inf()) : av;
            bblk = given ? (bv > -1.0e29f ? bv * Num<float>::kLn2 : Num<float>::neg_inf()) : bv;
#pragma unroll
            for (int s = 1; s < 64; s <<= 1) {
                ablk = __builtin_fmaxf(ablk, __shfl_xor(ablk, s, 64));
                bblk = __builtin_fmaxf(bblk, __shfl_xor(bblk, s, 64));
            }
        }
        if (!(__builtin_fabsf(ablk) < 3.0e38f)) ablk = 0.0f; // (no finite entry, or an infinite one)
        if (!(__builtin_fabsf(bblk) < 3.0e38f)) bblk = 0.0f;
        constexpr float kPerUnit = 16.0f, kFloor = -4096.0f * 16.0f;
        // NaN counts as the largest, so that the output is looked at and comes out as NaN
        auto key_of = [&](float v, float top16) { return v == v ? __builtin_rintf(__builtin_amdgcn_fmed3f(__builtin_fmaf(v, kPerUnit, top16), kFloor, 0.0f)) : 0.0f; };
        const float atop16 = -kPerUnit * ablk, btop16 = -kPerUnit * bblk;
        struct Pair {
            float re, im;
        };
        // entry u of a thread: A'[2 u + tid / 128][tid % 128] and B'[4 u + tid / 64][tid % 64] of the block, so that a
        // wave reads 512 consecutive bytes at a time and a thread's entries lie a fixed stride apart.  The signs of a
        // thread's 32 entries of an operand make one word (bit u), stored under the thread's number.
        float ha[kHeld], hb[kHeld];
        unsigned sign_a = 0, sign_b = 0;
        const int ra0 = tid / kKeyedMaxInner, ja = tid % kKeyedMaxInner, jb0 = tid / kOut, cb = tid % kOut;
        auto stage_operands = [&](auto whole) __attribute__((always_inline)) {
            constexpr bool WHOLE = decltype(whole)::value; // the block lies inside the operands and d is 128: no edges
            // (WHOLE: one address for the wave, which moves on from entry to entry, and a thread's 32-bit offset from it)
            const float *base_a = Ab + (size_t)i0 * d * 2, *base_b = Bb + (size_t)k0 * 2;
            const unsigned off_a = ((unsigned)ra0 * (unsigned)d + (unsigned)ja) * 2u, off_b = ((unsigned)jb0 * (unsigned)m + (unsigned)cb) * 2u;
            const size_t step_a = (size_t)4 * d, step_b = (size_t)8 * m; // floats from one entry to the next
#pragma unroll
            for (int u0 = 0; u0 < kHeld; u0 += 16) {
                Pair va[16], vb[16]; // sixteen loads of each in flight
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    if constexpr (WHOLE) {
                        va[u] = *reinterpret_cast<const Pair *>(base_a + (u0 + u) * step_a + off_a);
                        vb[u] = *reinterpret_cast<const Pair *>(base_b + (u0 + u) * step_b + off_b);
                    } else { // (from addresses held inside the operands)
                        const int r = 2 * (u0 + u) + ra0, jb = 4 * (u0 + u) + jb0;
                        va[u] = *reinterpret_cast<const Pair *>(Ab + ((size_t)(i0 + r < n ? i0 + r : n - 1) * d + (ja < d ? ja : d - 1)) * 2);
                        vb[u] = *reinterpret_cast<const Pair *>(Bb + ((size_t)(jb < d ? jb : d - 1) * m + (k0 + cb < m ? k0 + cb : m - 1)) * 2);
                    }
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const int r = 2 * (u0 + u) + ra0, jb = 4 * (u0 + u) + jb0;
                    const bool ina = WHOLE || (i0 + r < n && ja < d), inb = WHOLE || (k0 + cb < m && jb < d);
                    const float xa = ina ? va[u].re : Num<float>::neg_inf(), xb = inb ? vb[u].re : Num<float>::neg_inf();
                    ha[u0 + u] = xa;
                    hb[u0 + u] = xb;
                    kx[r * kKeyedLda + ja] = key_of(xa, atop16); // (-inf gets the lowest key)
                    ky[jb * kOut + cb] = key_of(xb, btop16) + (float)jb * (1.0f / kKeyedMaxInner);
                    sign_a |= (ina ? (unsigned)Num<float>::parity(va[u].im) : 0u) << (u0 + u);
                    sign_b |= (inb ? (unsigned)Num<float>::parity(vb[u].im) : 0u) << (u0 + u);
                }
            }
        };
        if (d == kKeyedMaxInner && i0 + kOut <= n && k0 + kOut <= m)
            stage_operands(std::true_type{});
        else
            stage_operands(std::false_type{});
        sa[tid] = sign_a;
        sb[tid] = sign_b;
        __syncthreads();
        float k1[4][4], k2[4][4], k3[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) k1[r][c] = k2[r][c] = k3[r][c] = -3.0e6f;
        // (The largest of two as a median with +inf, handed over as a kernel argument: one instruction, where the plain
        // maximum would first put its operand in canonical form.)
        const float inf = a.pos_inf;
#pragma unroll 4
        for (int j = 0; j < kKeyedMaxInner; ++j) {
            float x[4], y[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) x[r] = kx[(4 * ty + r) * kKeyedLda + j];
#pragma unroll
            for (int c = 0; c < 4; ++c) y[c] = ky[j * kOut + 4 * tx + c];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float key = x[r] + y[c];
                    k3[r][c] = __builtin_amdgcn_fmed3f(k2[r][c], k3[r][c], key);
                    k2[r][c] = __builtin_amdgcn_fmed3f(k1[r][c], k2[r][c], key);
                    k1[r][c] = __builtin_amdgcn_fmed3f(k1[r][c], key, inf);
                }
        }
        // ---- the operands in the keys' place
        float *xf = kx, *yf = ky;
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kHeld; ++u) {
            xf[(2 * u + ra0) * kKeyedLda + ja] = ha[u];
            yf[(4 * u + jb0) * kOut + cb] = hb[u];
        }
        if (tid == 0) s_count = 0;
        __syncthreads();
        // the two leading terms of every output, exactly, by the indices their keys carry
        auto term = [&](int il, int kl, float key, float &t, unsigned &neg) {
            const int j = (int)(key * (float)kKeyedMaxInner) & (kKeyedMaxInner - 1);
            t = xf[il * kKeyedLda + j] + yf[j * kOut + kl];
            neg = ((sa[(il % 2) * kKeyedMaxInner + j] >> (il / 2)) ^ (sb[(j % 4) * kOut + kl] >> (j / 4))) & 1u;
        };
        const float base = ablk + bblk;
        // All d terms but the leading ones, each at most what the next key says, may be left out when together they
        // move the result's logarithm by less than a quarter of its last place, |result| 2^-26: their share of the sum
        // below that.  (A key understates its term by at most 1/16: two roundings to 1/32.)
        const float slack0 = ::logf((float)d) + 0.07f + 26.0f * Num<float>::kLn2;
        auto slack = [&](float result) { return slack0 - __builtin_amdgcn_logf(__builtin_fmaxf(__builtin_fabsf(result), 2.0f)) * Num<float>::kLn2; };
        unsigned full = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float t1[4], t2[4];
            unsigned s1[4], s2[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                term(4 * ty + r, 4 * tx + c, k1[r][c], t1[c], s1[c]);
                term(4 * ty + r, 4 * tx + c, k2[r][c], t2[c], s2[c]);
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const float b2 = k2[r][c] * (1.0f / kPerUnit) + base, b3 = k3[r][c] * (1.0f / kPerUnit) + base;
                const float hi = __builtin_fmaxf(t1[c], t2[c]), lo = __builtin_fminf(t1[c], t2[c]);
                const float e = __builtin_amdgcn_exp2f((lo - hi) * Num<float>::kLog2e); // in (0, 1]
                const float w = s1[c] == s2[c] ? 1.0f + e : 1.0f - e;
                const float both = hi + __builtin_amdgcn_logf(w) * Num<float>::kLn2; // (w is no denormal number that matters)
                float re_out, im_out;
                bool done = false;
                if (b2 + slack(t1[c]) < t1[c]) { // one term decides
                    re_out = t1[c];
                    im_out = s1[c] ? Num<float>::pi() : 0.0f;
                    done = true;
                } else if (w > 0.0f && b3 + slack(both) < both) { // two terms decide, also after cancellation between them
                    re_out = both;
                    im_out = (t1[c] >= t2[c] ? s1[c] : s2[c]) ? Num<float>::pi() : 0.0f;
                    done = true;
                }
                if (need & (1u << (4 * r + c))) {
                    if (done) {
                        *reinterpret_cast<Pair *>(Cb + ((size_t)(i0 + 4 * ty + r) * m + k0 + 4 * tx + c) * 2) = Pair{re_out, im_out};
                    } else {
                        full |= 1u << (4 * r + c);
                    }
                }
            }
        }
        // the outputs still open, as a list: a wave reserves room for all of its lanes' at once
        {
            const int lane = tid & 63, mine = __builtin_popcount(full);
            int before = mine; // inclusive prefix sum over the wave
#pragma unroll
            for (int s = 1; s < 64; s <<= 1) {
                const int o = __shfl_up(before, s, 64);
                if (lane >= s) before += o;
            }
            int first = 0;
            if (lane == 63 && before > 0) first = atomicAdd(&s_count, before);
            first = __shfl(first, 63, 64);
            int slot = first + before - mine;
            for (unsigned rest = full; rest != 0; rest &= rest - 1) {
                const int q = __builtin_ctz(rest);
                open[slot++] = (unsigned short)((4 * ty + q / 4) * kOut + 4 * tx + q % 4);
            }
        }
        __syncthreads();
        const int nopen = s_count;
        // ---- a lane takes one of them and walks the inner index twice (largest term, then the sum)
        for (int e = tid; e < nopen; e += kThreads) {
            const int il = open[e] / kOut, kl = open[e] % kOut;
            const float *xr = xf + il * kKeyedLda, *yc = yf + kl;
            float zmax = Num<float>::neg_inf();
#pragma unroll 8
            for (int j = 0; j < kKeyedMaxInner; ++j) zmax = __builtin_fmaxf(zmax, xr[j] + yc[j * kOut]);
            const float scale = zmax > Num<float>::neg_inf() ? -(zmax * Num<float>::kLog2e) : 0.0f;
            float sv = 0.0f;
            const unsigned *sar = sa + (il % 2) * kKeyedMaxInner, *sbc = sb + kl;
#pragma unroll 8
            for (int j = 0; j < kKeyedMaxInner; ++j) {
                const float t = Num<float>::exp2_(Num<float>::fma_(xr[j] + yc[j * kOut], Num<float>::kLog2e, scale));
                const unsigned flip = ((sar[j] >> (il / 2)) ^ (sbc[(j % 4) * kOut] >> (j / 4))) << 31;
                sv += __builtin_bit_cast(float, __builtin_bit_cast(unsigned, t) ^ flip);
            }
            float *out = Cb + ((size_t)(i0 + il) * m + k0 + kl) * 2;
            *reinterpret_cast<Pair *>(out) = Pair{sv != 0.0f ? (::log2f(__builtin_fabsf(sv)) - scale) * Num<float>::kLn2 : Num<float>::neg_inf(),
                                                  sv < 0.0f ? Num<float>::pi() : 0.0f};
        }
        return;
    }
    // ---- many outputs to repair: first the largest pairwise sum of every output of the block ...
    R mx[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) mx[r][c] = Num<R>::neg_inf();
    for (int j0 = 0; j0 < d; j0 += kJBlock) {
        stage(j0);
#pragma unroll 4
        for (int j = 0; j < kJBlock; ++j) {
            R x[4], y[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) x[r] = are[(4 * ty + r) * LDA + j];
#pragma unroll
            for (int c = 0; c < 4; ++c) y[c] = bre[j * kOut + 4 * tx + c];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) mx[r][c] = Num<R>::max_(x[r] + y[c], mx[r][c]);
        }
    }
    // ---- ... then the signed sums of exponentials relative to it.  Every thread stages; a wave none of
    // whose outputs needs repair skips the arithmetic.
    const bool wave_needs = __builtin_amdgcn_ballot_w64(need != 0) != 0;
    // which of the sixteen output positions any lane of this wave has to repair: when repairs are rare
    // (double components), most positions are skipped by the whole wave
    unsigned wave_mask = 0;
#pragma unroll
    for (int q = 0; q < 16; ++q)
        if (__builtin_amdgcn_ballot_w64((need >> q) & 1u) != 0) wave_mask |= 1u << q;
    // A term is 2^((x + y) log2(e) + nmx) with nmx = -(mx log2(e)), rounded: one fused multiply-add, whose exponent
    // is exact, so the sum is the true one times 2^nmx whatever the rounding of nmx, and the result is
    // (log2|sum| - nmx) ln 2.  (An output with no finite term has all terms zero and stays at -inf.)
    R sum[4][4], nmx[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            sum[r][c] = 0;
            const R mxl = mx[r][c] > Num<R>::neg_inf() ? mx[r][c] : (R)0;
            nmx[r][c] = -(mxl * Num<R>::kLog2e);
        }
    // one block of j; ALL: every position is wanted by some lane (wide-range float data), so the sixteen
    // wave-uniform tests per inner index are left out
    auto sweep_block = [&](auto all) __attribute__((always_inline)) {
        constexpr bool ALL = decltype(all)::value;
#pragma unroll 2
        for (int j = 0; j < kJBlock; ++j) {
            R x[4], y[4];
            float sx[4], sy[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                x[r] = are[(4 * ty + r) * LDA + j];
                sx[r] = asg[(4 * ty + r) * LDA + j];
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                y[c] = bre[j * kOut + 4 * tx + c];
                sy[c] = bsg[j * kOut + 4 * tx + c];
            }
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (ALL || (wave_mask & (1u << (4 * r + c)))) {
                        const R t = Num<R>::exp2_(Num<R>::fma_(x[r] + y[c], Num<R>::kLog2e, nmx[r][c]));
                        sum[r][c] = Num<R>::fma_(t, flip_sign<R>((R)sx[r], sy[c]), sum[r][c]);
                    }
        }
    };
    for (int j0 = 0; j0 < d; j0 += kJBlock) {
        if (d > kJBlock) stage(j0); // a single block of j is still in LDS
        if (wave_needs) {
            if constexpr (sizeof(R) == 4) { // (double components: repairs are rare, and a second copy of the loop costs registers)
                if (wave_mask == 0xffffu)
                    sweep_block(std::true_type{});
                else
                    sweep_block(std::false_type{});
            } else {
                sweep_block(std::false_type{});
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (need & (1u << (4 * r + c))) {
                const int i = i0 + 4 * ty + r, k = k0 + 4 * tx + c;
                R re_out = Num<R>::neg_inf(), im_out = 0;
                const R sv = sum[r][c];
                if (sv != 0) {
                    re_out = (Num<R>::log2_(sv < 0 ? -sv : sv) - nmx[r][c]) * Num<R>::kLn2;
                    im_out = sv < 0 ? Num<R>::pi() : (R)0;
                }
                Cb[((size_t)i * m + k) * 2] = re_out;
                Cb[((size_t)i * m + k) * 2 + 1] = im_out;
            }
    };
#pragma unroll 1
    for (int sb = 0; sb < (kSuper / kOut) * (kSuper / kOut); ++sb) {
        const int si = sb / (kSuper / kOut), sk = sb % (kSuper / kOut);
        i0 = I0 + si * kOut;
        k0 = K0 + sk * kOut;
        if (i0 < n && k0 < m) repair_block(s_amax + si * kOut, s_bmax + sk * kOut); // (the same for every thread)
    }
}

} // namespace

namespace goom {

int launch_lmme_exact(goom_ctx *ctx, const void *A, const void *B, void *C, long long batch, int n, int d, int m, int dtype,
                      const void *shifts)
{
    if (shifts && (n != 128 || m != 128)) return fail(ctx, GOOM_EINVAL, "shifts are handed over for 128 x 128 outputs only");
    ExactArgs a;
    a.A = A;
    a.B = B;
    a.C = C;
    a.shifts = shifts;
    a.batch = batch;
    a.n = n;
    a.d = d;
    a.m = m;
    a.pos_inf = __builtin_huge_valf();
    const int sup = dtype == GOOM_C64 ? super_block<float>() : super_block<double>();
    const long long grid = batch * ((n + sup - 1) / sup) * ((m + sup - 1) / sup);
    if (grid > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "too many output blocks for one launch");
    const size_t comp = dtype == GOOM_C64 ? 4 : 8;
    const bool keyed = dtype == GOOM_C64 && d <= kKeyedMaxInner && (long long)n * m < (1LL << 28);
    size_t lds = (size_t)kOut * (kJBlock + 1) * (comp + 4) + (size_t)kJBlock * kOut * (comp + 4) + 64;
    if (keyed && lds < kKeyedLds) lds = kKeyedLds;
    const void *kern = dtype != GOOM_C64 ? reinterpret_cast<const void *>(lmme_exact_kernel<double, false>)
                       : keyed           ? reinterpret_cast<const void *>(lmme_exact_kernel<float, true>)
                                         : reinterpret_cast<const void *>(lmme_exact_kernel<float, false>);
    if (lds > 48 * 1024) {
        if (int st = check_hip(ctx, hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds), "hipFuncSetAttribute(lmme_exact_kernel)")) return st;
    }
    prof_begin(ctx, "lmme_exact_repair");
    if (dtype != GOOM_C64)
        hipLaunchKernelGGL((lmme_exact_kernel<double, false>), dim3((unsigned)grid), dim3(kThreads), lds, ctx->stream, a);
    else if (keyed)
        hipLaunchKernelGGL((lmme_exact_kernel<float, true>), dim3((unsigned)grid), dim3(kThreads), lds, ctx->stream, a);
    else
        hipLaunchKernelGGL((lmme_exact_kernel<float, false>), dim3((unsigned)grid), dim3(kThreads), lds, ctx->stream, a);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch lmme_exact_kernel");
}

} // namespace goom
