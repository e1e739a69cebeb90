// Carry phase of the selectively reset scan (paper Section 5; Section 4.2.1 item (a)).
//
// The reset scan cuts the chain into chunks like the plain scan.  Phase 1 (chain kernel)
// multiplies every chunk down to one factored matrix T_c.  This kernel is phase 2: one
// workgroup per batch item walks the chunks in order, keeping the true prefix state
//     Z = T_c Y_c            (the state at step (c + 1) L),
// examines it with the selection function S (always / near-colinear columns / never), and
// when selected replaces it by R(Z): columns scaled to unit norm, then the orthonormal
// factor Q of a QR factorisation with positive diagonal.  The prefix that enters chunk
// c + 1, Y_{c+1}, is written for phase 3 (chain kernel), which re-walks every chunk and
// stores all states.  Because S and R are applied only to true prefix states, left to
// right, the result does not depend on a scan tree: it is the sequential recurrence with
// its states examined every L steps.
//
// Per column k a reset removes log R_kk + log(norm of column k) of log-growth from the
// state; these accumulate (in double) into growth[k], plus the same quantities for the
// final state, so growth / (dt T) is the Lyapunov spectrum (paper Section 4.2.1, eq. 20, with the
// triangular factors taken at the resets: triangular factors multiply, so their diagonals
// accumulate exactly as in the step-by-step method).
//
// One wave per batch item, matrices in registers, float arithmetic with double accumulation
// of the logarithms.  The chain of chunks is inherently serial (each reset depends on the
// previous one), so this phase is latency bound: what counts is the length of the dependent
// instruction chain per chunk, which is why it runs without a single workgroup barrier.
#include <cstring>

#include "goom_internal.h"

namespace {

constexpr double kLn2 = 0.693147180559945309417;
constexpr double kLog2e = 1.44269504088896340736;
constexpr int kThreads = 256;

struct ResetArgs {
    const unsigned char *totals; // [batch][C] factored chunk products (common exponent), DP x tot_cols
    long long tot_stride;
    int tot_cols;
    unsigned char *carries;      // [batch][C + 1] factored prefixes entering each chunk (and the final state), DP x car_cols
    long long car_stride;
    int car_cols;
    const void *s0;              // NULL or GOOM initial state [batch][d][d] (complex64 or complex128)
    unsigned char *chunk_flags;  // [batch][C]: 1 where the state at the end of chunk c was reset
    double *growth;              // NULL or [batch][d]
    double growth_scale;         // 1, or 1 / (dt T) to return exponents
    long long T, L, C;
    int d;
    int policy;
    float cos_threshold;
};

typedef float f4 __attribute__((ext_vector_type(4)));

__device__ inline f4 mfma4(float x, float y, f4 acc) { return __builtin_amdgcn_mfma_f32_16x16x4f32(x, y, acc, 0, 0, 0); }

__device__ inline float read_lane(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// LDS operations of one wave complete in program order; this only keeps the compiler from
// moving them across the point where lanes hand data to each other.
__device__ inline void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

typedef double d4 __attribute__((ext_vector_type(4)));

// One wave per batch item.  All DP x DP matrices live in registers in the layout the
// 16 x 16 x 4 matrix instruction leaves its result in: lane (g = lane / 16, c = lane % 16),
// register [nt][mt][v] holds entry (row 16 mt + 4 g + v, column 16 nt + c).  That layout is
// also the instruction's B operand, and, read as "column block first", the A operand of the
// transpose, so both Z = T Y and the Gram matrix G = Z^T Z run on the matrix unit without
// moving the state; only the chunk product T goes through LDS (it arrives row by row).
//
// QR by the Gram matrix: Cholesky elimination G = R^T R, one column per step, with the same
// column operations applied to Z, which turns Z into Q = Z R^-1 in place; row k of G and
// column k of Z reach the other lanes through a few words of LDS.  The pivots are the
// squares of R's diagonal.  G is formed and eliminated in double (the double-precision
// matrix instruction; its result has row 16 mt + 4 v + g in register v), so the pivots stay
// accurate up to cond(Z)^2 of about 1e12; the columns of Z are updated in float, which
// costs orthogonality in proportion to sqrt(largest ratio of a column's squared norm to its
// pivot).  When that ratio is large the factorisation is repeated on Q, which restores
// orthogonality to rounding level, and the two diagonals multiply.
template <int DP> struct Wave {
    static constexpr int KT = DP / 16;
    static constexpr int LDT = DP + 4;
    float tile[DP * LDT]; // chunk product, row-major, rows padded against bank conflicts
    double rrow[2][DP];   // row k of G at step k, entry j at position j (two sets, used alternately)
    double rperm[2][DP];  // the same with entry 16 mt + 4 v + g at position 16 mt + 4 g + v
    float qcol[2][DP];    // column k of Z at step k
    double diag[DP];      // diagonal of the Gram matrix
    float qpanel[DP / 16][DP * 20]; // finished panels of Q, [row][column within the panel], rows padded to 20
};

// The factorisation runs panel by panel (16 columns at a time), in square-root-free form: a step
// subtracts (G_kj / p_k) times row / column k from every later one of the panel, p_k = G_kk being the
// pivot, and the columns are scaled by 1 / sqrt(p) at the end of the panel.  The row and the column of
// step k go to LDS as they are, so their round trip overlaps with the reciprocal of the pivot, the
// other half of the dependent chain.  A panel is first made orthogonal to the finished panels on the matrix unit (R_qp = Q_q^T Z_p, then
// Z_p -= Q_q R_qp: the first product reads both operands in place, the second takes Q_q from LDS as
// its left operand and R_qp, as the matrix instruction left it, as its right operand), then its own
// 16 x 16 Gram matrix is eliminated as above.  A step then touches 16 columns instead of all of
// them, and only one 16 x 16 tile of G is alive at a time.

// elimination of one panel: G is its 16 x 16 Gram matrix (register v = row 4 v + g, column c),
// Zp its columns; pivots to piv for the lanes that own the column
template <int DP> __device__ void eliminate_panel(d4 &G, f4 (&Zp)[DP / 16], double &piv, Wave<DP> &s, int g, int c)
{
    constexpr int KT = DP / 16;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const int gk = k % 4, vk = k / 4; // row k of G: lanes with g == gk, register vk
        const int buf = k & 1;
        double *rrow = s.rrow[buf];
        double *rperm = s.rperm[buf];
        float *qcol = s.qcol[buf];
        if (g == gk) {
            const double r = c > k ? G[vk] : 0.0; // zero left of the diagonal: finished columns stay put
            rrow[c] = r;
            rperm[((c & 3) << 2) | (c >> 2)] = r;
        }
        if (c == k) {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) *reinterpret_cast<f4 *>(&qcol[16 * mt + 4 * g]) = Zp[mt];
        }
        const double pv = G[vk];
        const int lo = __builtin_amdgcn_readlane((int)(__builtin_bit_cast(unsigned long long, pv) & 0xffffffffull), 16 * gk + k);
        const int hi = __builtin_amdgcn_readlane((int)(__builtin_bit_cast(unsigned long long, pv) >> 32), 16 * gk + k);
        const double pivot = __builtin_bit_cast(double, ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo);
        if (c == k) piv = pivot;
        const bool live = pivot > 1.0e-30;
        const double r0 = (double)__builtin_amdgcn_rcpf((float)pivot);
        const double inv = live ? r0 * (2.0 - pivot * r0) : 0.0;
        wave_sync();
        const double tj = rrow[c] * inv;
        const d4 ri = *reinterpret_cast<const d4 *>(&rperm[4 * g]); // rows 4 v + g, v = 0..3
        G -= ri * tj;
        const float tjf = (float)tj;
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) {
            const f4 zk = *reinterpret_cast<const f4 *>(&qcol[16 * mt + 4 * g]);
            Zp[mt] -= zk * tjf;
        }
    }
    wave_sync();
}

// QR of Z in place (Z <- Q), panel by panel; piv[nt] = squared diagonal of R for column 16 nt + c.
// Returns the largest ratio (squared column norm) / pivot, a measure of cond(Z)^2.
template <int DP> __device__ float qr_panels(f4 (&Z)[DP / 16][DP / 16], double (&piv)[DP / 16], Wave<DP> &s, int g, int c)
{
    constexpr int KT = DP / 16;
    float norm2[KT];
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) {
        float a = 0.0f;
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) a = __builtin_fmaf(Z[nt][mt][v], Z[nt][mt][v], a);
        a += __shfl_xor(a, 16, 64);
        a += __shfl_xor(a, 32, 64);
        norm2[nt] = a;
    }
#pragma unroll
    for (int p = 0; p < KT; ++p) {
        // orthogonal to the finished panels; twice, because one float projection leaves about
        // 2^-24 of the panel's norm behind, which the panel's own (much smaller) remainder would magnify
#pragma unroll
        for (int rep = 0; rep < (p > 0 ? 2 : 0); ++rep)
#pragma unroll
        for (int q = 0; q < p; ++q) {
            f4 R = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int v = 0; v < 4; ++v) R = mfma4(Z[q][kt][v], Z[p][kt][v], R);
            R = -R;
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                const f4 av = *reinterpret_cast<const f4 *>(&s.qpanel[q][(16 * mt + c) * 20 + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v) Z[p][mt] = mfma4(av[v], R[v], Z[p][mt]);
            }
        }
        // the panel's own Gram matrix, in double
        d4 G = {0., 0., 0., 0.};
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) G = __builtin_amdgcn_mfma_f64_16x16x4f64((double)Z[p][kt][v], (double)Z[p][kt][v], G, 0, 0, 0);
        piv[p] = 1.0;
        eliminate_panel<DP>(G, Z[p], piv[p], s, g, c);
        const bool live = piv[p] > 1.0e-30;
        const float sc = live ? __builtin_amdgcn_rsqf((float)piv[p]) : 0.0f;
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) Z[p][mt] *= sc;
        if (p + 1 < KT) {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v) s.qpanel[p][(16 * mt + 4 * g + v) * 20 + c] = Z[p][mt][v];
            wave_sync();
        }
    }
    float worst = 1.0f;
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) {
        const float ratio = piv[nt] > 1.0e-30 ? norm2[nt] * __builtin_amdgcn_rcpf((float)piv[nt]) : 1.0f;
        worst = fmaxf(worst, ratio);
    }
#pragma unroll
    for (int sft = 1; sft < 16; sft <<= 1) worst = fmaxf(worst, __shfl_xor(worst, sft, 64));
    return read_lane(worst, 0); // the same in every lane; this tells the compiler so
}

// ---------------------------------------------------------------------------------------------------
// The carry kernel keeps everything in double: the chunk products arrive in double, Z = T Y and every step
// of the factorisation run on the double-precision matrix instruction and the double vector ALU.  The
// 16 x 16 x 4 double instruction leaves rows 4 v + g of column c in register v of lane (g, c), takes
// A[row c][k = g] and B[k = g][column c] from lane (g, c); so a matrix held as [nt][mt] tiles in that result
// layout is, register for register, a B operand whose contraction index runs 4 v + g, and an A operand of
// its transpose.  Whatever is read from LDS as a four-vector therefore stores index 4 v + g at position
// 4 g + v (perm16 below).
__device__ inline int perm16(int j) { return (j & ~15) | ((j & 3) << 2) | ((j >> 2) & 3); }

template <int DP> struct WaveD {
    static constexpr int LDT = DP + 2;  // row stride of the chunk product (doubles)
    static constexpr int LDQ = 18;      // row stride of a finished panel
    double tile[DP * LDT]; // chunk product, rows in order, columns in perm16 order
    double rrow[2][16];   // row k of the panel's Gram matrix at step k, entry j at position j
    double rperm[2][16];  // the same in perm16 order
    double qcol[2][DP];   // column k of the panel at step k, rows in perm16 order
    double diag[DP];      // diagonal of the Gram matrix (selection by cosines)
    // blocked elimination (panels of up to 32 rows only): the four pivot rows of a block, entry j at position j; the
    // same in perm16 order; the four pivot columns of the panel, rows in perm16 order
    double brow[DP <= 32 ? 4 : 1][16];
    double bperm[DP <= 32 ? 4 : 1][16];
    double bcol[DP <= 32 ? 4 : 1][DP];
    double qpanel[DP / 16 > 1 ? DP / 16 - 1 : 1][DP * LDQ]; // finished panels of Q: [row][column within the panel, perm16 order]
};

__device__ inline d4 mfma8(double x, double y, d4 acc) { return __builtin_amdgcn_mfma_f64_16x16x4f64(x, y, acc, 0, 0, 0); }

__device__ inline double read_lane_d(double v, int lane)
{
    const unsigned long long u = __builtin_bit_cast(unsigned long long, v);
    const int lo = __builtin_amdgcn_readlane((int)(u & 0xffffffffull), lane);
    const int hi = __builtin_amdgcn_readlane((int)(u >> 32), lane);
    return __builtin_bit_cast(double, ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo);
}

// 1 / x and 1 / sqrt(x) to double precision from the float hardware approximations (x within float range)
__device__ inline double rcp_d(double x)
{
    double r = (double)__builtin_amdgcn_rcpf((float)x);
    r = r * (2.0 - x * r);
    return r * (2.0 - x * r);
}
__device__ inline double rsqrt_d(double x)
{
    double r = (double)__builtin_amdgcn_rsqf((float)x);
    r = r * (1.5 - 0.5 * x * r * r);
    return r * (1.5 - 0.5 * x * r * r);
}

// elimination of one panel (see eliminate_panel above), columns in double
template <int DP, typename S> __device__ void eliminate_panel_d(d4 &G, d4 (&Zp)[DP / 16], double &piv, S &s, int g, int c)
{
    constexpr int KT = DP / 16;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const int gk = k % 4, vk = k / 4;
        const int buf = k & 1;
        double *rrow = s.rrow[buf];
        double *rperm = s.rperm[buf];
        double *qcol = s.qcol[buf];
        if (g == gk) {
            const double r = c > k ? G[vk] : 0.0;
            rrow[c] = r;
            rperm[((c & 3) << 2) | (c >> 2)] = r;
        }
        if (c == k) {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) *reinterpret_cast<d4 *>(&qcol[16 * mt + 4 * g]) = Zp[mt];
        }
        const double pivot = read_lane_d(G[vk], 16 * gk + k);
        if (c == k) piv = pivot;
        const double inv = pivot > 1.0e-280 ? rcp_d(pivot) : 0.0;
        wave_sync();
        const double tj = rrow[c] * inv;
        const d4 ri = *reinterpret_cast<const d4 *>(&rperm[4 * g]);
        G -= ri * tj;
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) {
            const d4 zk = *reinterpret_cast<const d4 *>(&qcol[16 * mt + 4 * g]);
            Zp[mt] -= zk * tj;
        }
    }
    wave_sync();
}

// The same elimination four pivots at a time (panels of up to 32 rows): the four pivot rows of the Gram matrix and
// the four pivot columns of the panel make one trip through LDS, and every lane then carries out the four steps on
// copies of its own (the 4 x 4 block on the diagonal, the pivot rows at its own column and at the columns whose
// numbers are its rows', the pivot columns at its rows): the same multiply-adds on the same numbers in the same
// order as one pivot at a time, four times fewer waits for LDS.
template <int DP> __device__ void eliminate_panel_blocked(d4 &G, d4 (&Zp)[DP / 16], double &piv, WaveD<DP> &s, int g, int c)
{
    constexpr int KT = DP / 16;
    const int pc = ((c & 3) << 2) | (c >> 2);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        wave_sync();
        // row 4 b + g of the Gram matrix at column c; columns 4 b + j of the panel (from the lanes that hold them)
        s.brow[g][c] = G[b];
        s.bperm[g][pc] = G[b];
        if ((c >> 2) == b) {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) *reinterpret_cast<d4 *>(&s.bcol[c & 3][16 * mt + 4 * g]) = Zp[mt];
        }
        wave_sync();
        double a[4];   // pivot row j at this lane's column
        d4 P[4];       // pivot row j at columns 4 v + g
        d4 B[4];       // pivot row j at columns 4 b + i
        d4 zb[4][KT];  // pivot column j at this lane's rows
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            a[j] = s.brow[j][c];
            P[j] = *reinterpret_cast<const d4 *>(&s.bperm[j][4 * g]);
            B[j] = *reinterpret_cast<const d4 *>(&s.brow[j][4 * b]);
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) zb[j][mt] = *reinterpret_cast<const d4 *>(&s.bcol[j][16 * mt + 4 * g]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int k = 4 * b + j;
            const double pivot = B[j][j];
            if (c == k) piv = pivot;
            const double inv = pivot > 1.0e-280 ? rcp_d(pivot) : 0.0;
            // row k beyond the pivot, as the one-pivot form stores it: zero up to and including column k
            const double rc = c > k ? a[j] : 0.0;
            const double tj = rc * inv;
            d4 ri;
#pragma unroll
            for (int v = 0; v < 4; ++v) ri[v] = (4 * v + g > k) ? P[j][v] : 0.0;
            const d4 rinv = ri * inv; // (row k times 1 / pivot: the multipliers of the columns 4 v + g)
            G -= ri * tj;
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) Zp[mt] -= zb[j][mt] * tj;
            // the later pivot rows and columns of the block, brought up to date the same way
#pragma unroll
            for (int i = j + 1; i < 4; ++i) {
                const double rki = B[j][i];         // row k at column 4 b + i (> k)
                const double ti = rki * inv;        // the multiplier of column 4 b + i
                a[i] -= rki * tj;                   // entry (4 b + i, c): row factor times this column's multiplier
                P[i] -= rinv * rki;                 // entries (4 b + i, 4 v + g): row factor times those columns' multipliers
#pragma unroll
                for (int i2 = j + 1; i2 < 4; ++i2) B[i][i2] -= rki * (B[j][i2] * inv);
#pragma unroll
                for (int mt = 0; mt < KT; ++mt) zb[i][mt] -= zb[j][mt] * ti;
            }
        }
    }
    wave_sync();
}

// QR of Z in place (Z <- Q), panel by panel; piv[nt] = squared diagonal of R for column 16 nt + c.  Returns the
// largest ratio (squared column norm) / pivot, a measure of cond(Z)^2.  Before the factorisation every column
// is scaled by a power of two to a largest entry near 1 (cexp receives the exponents), so that pivots stay
// inside the range of the float reciprocal estimates.
template <int DP> __device__ double qr_panels_d(d4 (&Z)[DP / 16][DP / 16], double (&piv)[DP / 16], double (&cexp)[DP / 16], WaveD<DP> &s, int g, int c)
{
    constexpr int KT = DP / 16;
    constexpr int LDQ = WaveD<DP>::LDQ;
    double norm2[KT];
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) {
        double mx = 0.0;
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) mx = fmax(mx, fabs(Z[nt][mt][v]));
        mx = fmax(mx, __shfl_xor(mx, 16, 64));
        mx = fmax(mx, __shfl_xor(mx, 32, 64));
        int ex = 0;
        if (mx > 0.0) (void)frexp(mx, &ex);
        cexp[nt] = (double)ex;
        double a = 0.0;
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                Z[nt][mt][v] = ldexp(Z[nt][mt][v], -ex);
                a = fma(Z[nt][mt][v], Z[nt][mt][v], a);
            }
        a += __shfl_xor(a, 16, 64);
        a += __shfl_xor(a, 32, 64);
        norm2[nt] = a;
    }
#pragma unroll
    for (int p = 0; p < KT; ++p) {
        // orthogonal to the finished panels (twice: one projection leaves rounding-level remainders of the
        // panel's norm behind, which the panel's own, much smaller, remainder would magnify)
#pragma unroll
        for (int rep = 0; rep < (p > 0 ? 2 : 0); ++rep)
#pragma unroll
            for (int q = 0; q < p; ++q) {
                d4 R = {0., 0., 0., 0.};
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) R = mfma8(Z[q][kt][v], Z[p][kt][v], R);
                R = -R;
#pragma unroll
                for (int mt = 0; mt < KT; ++mt) {
                    const d4 av = *reinterpret_cast<const d4 *>(&s.qpanel[q][(16 * mt + c) * LDQ + 4 * g]);
#pragma unroll
                    for (int v = 0; v < 4; ++v) Z[p][mt] = mfma8(av[v], R[v], Z[p][mt]);
                }
            }
        d4 G = {0., 0., 0., 0.};
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) G = mfma8(Z[p][kt][v], Z[p][kt][v], G);
        piv[p] = 1.0;
        if constexpr (DP <= 32)
            eliminate_panel_blocked<DP>(G, Z[p], piv[p], s, g, c);
        else
            eliminate_panel_d<DP>(G, Z[p], piv[p], s, g, c);
        const double sc = piv[p] > 1.0e-280 ? rsqrt_d(piv[p]) : 0.0;
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) Z[p][mt] *= sc;
        if (p + 1 < KT) {
#pragma unroll
            for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v) s.qpanel[p][(16 * mt + 4 * v + g) * LDQ + (((c & 3) << 2) | (c >> 2))] = Z[p][mt][v];
            wave_sync();
        }
    }
    double worst = 1.0;
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) {
        const double ratio = piv[nt] > 1.0e-280 ? norm2[nt] * rcp_d(piv[nt]) : 1.0;
        worst = fmax(worst, ratio);
    }
#pragma unroll
    for (int sft = 1; sft < 16; sft <<= 1) worst = fmax(worst, __shfl_xor(worst, sft, 64));
    return read_lane_d(worst, 0);
}

// IO: component type of the GOOM initial state (float for complex64, double for complex128)
template <int DP, typename IO> __global__ __launch_bounds__(64) void reset_carry_kernel(ResetArgs a)
{
    constexpr int KT = DP / 16;
    constexpr int LDT = WaveD<DP>::LDT;
    constexpr int TQ = DP * DP / 4 / 64; // 32-byte pieces (four doubles) of the chunk product per lane
    constexpr bool PREFETCH = DP <= 32;  // the next chunk product waits in registers during the factorisation
    __shared__ __align__(32) WaveD<DP> s;
    const int lane = threadIdx.x;
    const int g = lane >> 4, c = lane & 15;
    const int d = a.d;
    const long long b = blockIdx.x;
    const size_t tot_mant = (size_t)DP * a.tot_cols * sizeof(double);
    const size_t car_mant = (size_t)DP * a.car_cols * sizeof(double);

    d4 Y[KT][KT];    // state: Y[nt][mt][v] = entry (row 16 mt + 4 v + g, column 16 nt + c), columns scaled by 2^yexp
    double yexp[KT];
    double pprod[KT], pexp[KT]; // product of all pivots so far = pprod 2^pexp (column exponents counted twice: pivots are squares)
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) {
        yexp[nt] = 0.0;
        pprod[nt] = 1.0;
        pexp[nt] = 0.0;
    }
    // ---- initial state: identity or the given GOOM matrix; rows and columns past d carry an identity block,
    // which stays orthogonal to everything and never reaches the outputs
#pragma unroll
    for (int nt = 0; nt < KT; ++nt)
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) Y[nt][mt][v] = (16 * mt + 4 * v + g == 16 * nt + c) ? 1.0 : 0.0;
    if (a.s0) {
        const IO *gp = reinterpret_cast<const IO *>(a.s0) + (size_t)b * d * d * 2;
#pragma unroll
        for (int nt = 0; nt < KT; ++nt) {
            const int col = 16 * nt + c;
            if (col < d) {
                double cmax = -__builtin_huge_val();
                for (int i = 0; i < d; ++i) cmax = fmax(cmax, (double)gp[((size_t)i * d + col) * 2]);
                yexp[nt] = cmax > -__builtin_huge_val() ? ceil(cmax * kLog2e) : 0.0;
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = 16 * mt + 4 * v + g;
                        double val = 0.0;
                        if (row < d) {
                            const IO *e = gp + ((size_t)row * d + col) * 2;
                            const double t = (double)e[0] * kLog2e - yexp[nt];
                            val = t > -1000.0 ? exp2(t) : 0.0;
                            if ((int)rint((double)e[1] * 0.318309886183790671538) & 1) val = -val;
                        }
                        Y[nt][mt][v] = val;
                    }
            }
        }
    }

    auto store_carry = [&](long long cc) {
        unsigned char *dst = a.carries + (b * (a.C + 1) + cc) * a.car_stride;
        double *mp = reinterpret_cast<double *>(dst);
        double *ep = reinterpret_cast<double *>(dst + car_mant);
#pragma unroll
        for (int nt = 0; nt < KT; ++nt) {
            const int col = 16 * nt + c;
            if (col < a.car_cols) {
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = 16 * mt + 4 * v + g;
                        mp[(size_t)row * a.car_cols + col] = (row < d && col < d) ? Y[nt][mt][v] : 0.0;
                    }
                if (g == 0) ep[col] = col < d ? yexp[nt] : 0.0;
            }
        }
    };

    // chunk product cc: mantissas as pieces of four doubles (row = piece / (DP / 4)), and its common exponent
    auto total_ptr = [&](long long cc) { return a.totals + (b * a.C + cc) * a.tot_stride; };
    auto load_piece = [&](const unsigned char *tp, int q) {
        const int piece = lane + 64 * q;
        const int row = piece / (DP / 4), c4 = 4 * (piece % (DP / 4));
        return *reinterpret_cast<const d4 *>(reinterpret_cast<const double *>(tp) + (size_t)row * a.tot_cols + c4);
    };
    auto tile_piece = [&](double *tile, int q, d4 val) {
        const int piece = lane + 64 * q;
        const int row = piece / (DP / 4), c4 = 4 * (piece % (DP / 4));
        const int p4 = (c4 & ~15) | ((c4 >> 2) & 3);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            double x = val[e];
            if (row >= d || c4 + e >= d) x = (c4 + e == row) ? 1.0 : 0.0; // identity block past d
            tile[row * LDT + p4 + 4 * e] = x;
        }
    };

    // QR of Z in place (Z <- Q).  The growth it removes, ln R_kk + ln 2 * (exponent of column k), is kept as a
    // running product of pivots (mantissa and binary exponent apart) plus a sum of exponents, so that no logarithm
    // is taken inside the chain of chunks.
    auto qr_in_place = [&](d4 (&Z)[KT][KT], const double (&colexp)[KT]) {
        double piv[KT], piv2[KT], ce[KT], ce2[KT];
        const double amp = qr_panels_d<DP>(Z, piv, ce, s, g, c);
#pragma unroll
        for (int nt = 0; nt < KT; ++nt) {
            piv2[nt] = 1.0;
            ce2[nt] = 0.0;
        }
        // The factor Q comes out with errors of about amp 2^-53 relative to its columns' norms (amp: the squared
        // condition number).  For complex64 states, which are rounded to float, that is repaired by a second
        // factorisation from amp = 1e10 on; complex128 states take the second factorisation from 1e3 on.
        if (amp > (sizeof(IO) == 4 ? 1.0e10 : 1.0e3)) (void)qr_panels_d<DP>(Z, piv2, ce2, s, g, c);
#pragma unroll
        for (int nt = 0; nt < KT; ++nt)
            if (piv[nt] > 1.0e-280 && piv2[nt] > 1.0e-280) {
                int e;
                pprod[nt] = frexp(pprod[nt] * piv[nt] * piv2[nt], &e);
                pexp[nt] += 2.0 * (colexp[nt] + ce[nt] + ce2[nt]) + (double)e;
            }
    };

    d4 tq[PREFETCH ? TQ : 1];
    double tex_next = 0.0;
    if (PREFETCH && a.C > 0) {
        const unsigned char *tp = total_ptr(0);
        tex_next = *reinterpret_cast<const double *>(tp + tot_mant);
#pragma unroll
        for (int q = 0; q < TQ; ++q) tq[q] = load_piece(tp, q);
    }

    for (long long cc = 0; cc < a.C; ++cc) {
        store_carry(cc);
        double tex = tex_next;
        double *tile = s.tile;
        if (PREFETCH) {
#pragma unroll
            for (int q = 0; q < TQ; ++q) tile_piece(tile, q, tq[q]);
        } else { // (64-wide: the registers are taken by the state; the chunk product goes straight to LDS)
            const unsigned char *tp = total_ptr(cc);
            tex = *reinterpret_cast<const double *>(tp + tot_mant);
#pragma unroll 4
            for (int q = 0; q < TQ; ++q) tile_piece(tile, q, load_piece(tp, q));
        }
        wave_sync();
        if (PREFETCH && cc + 1 < a.C) {
            const unsigned char *tp = total_ptr(cc + 1);
            tex_next = *reinterpret_cast<const double *>(tp + tot_mant);
#pragma unroll
            for (int q = 0; q < TQ; ++q) tq[q] = load_piece(tp, q);
        }
        // ---- Z = T_c Y
        d4 Z[KT][KT];
#pragma unroll
        for (int nt = 0; nt < KT; ++nt)
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) Z[nt][mt] = d4{0., 0., 0., 0.};
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                const d4 av = *reinterpret_cast<const d4 *>(&tile[(16 * mt + c) * LDT + 16 * kt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int nt = 0; nt < KT; ++nt) Z[nt][mt] = mfma8(av[v], Y[nt][kt][v], Z[nt][mt]);
            }
        wave_sync(); // the tile is free again
        double zexp[KT];
#pragma unroll
        for (int nt = 0; nt < KT; ++nt) zexp[nt] = yexp[nt] + tex;

        const long long t_end = (cc + 1) * a.L; // 1-based step this chunk ends at (if it is a full chunk)
        const bool boundary = t_end <= a.T && a.policy >= 0;
        bool did_reset = false;
        if (boundary) {
            did_reset = a.policy == 1;
            if (!did_reset) {
                // squared cosines between columns, tile by tile of the Gram matrix: any pair above the threshold?
#pragma unroll
                for (int nt = 0; nt < KT; ++nt) {
                    d4 Gd = {0., 0., 0., 0.};
#pragma unroll
                    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                        for (int v = 0; v < 4; ++v) Gd = mfma8(Z[nt][kt][v], Z[nt][kt][v], Gd);
                    // G[j][j] for column j = 16 nt + c sits in lane (c % 4, c), register c / 4
                    double dsel = Gd[0];
                    dsel = (c >> 2) == 1 ? Gd[1] : dsel;
                    dsel = (c >> 2) == 2 ? Gd[2] : dsel;
                    dsel = (c >> 2) == 3 ? Gd[3] : dsel;
                    if (g == (c & 3)) s.diag[16 * nt + c] = dsel;
                }
                wave_sync();
                bool hit = false;
                const double thr2 = (double)a.cos_threshold * (double)a.cos_threshold;
#pragma unroll
                for (int nt = 0; nt < KT; ++nt) {
                    const double dc = s.diag[16 * nt + c];
#pragma unroll
                    for (int mt = 0; mt <= nt; ++mt) {
                        d4 Gt = {0., 0., 0., 0.}; // rows: columns 16 mt + .. of Z, columns: 16 nt + c
#pragma unroll
                        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                            for (int v = 0; v < 4; ++v) Gt = mfma8(Z[mt][kt][v], Z[nt][kt][v], Gt);
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int row = 16 * mt + 4 * v + g, col = 16 * nt + c;
                            const double dr = s.diag[row];
                            const double x = Gt[v];
                            if (row < col && col < d && x * x > thr2 * dr * dc) hit = true;
                        }
                    }
                }
                wave_sync();
                did_reset = __builtin_amdgcn_ballot_w64(hit) != 0;
            }
        }
        if (did_reset) {
            qr_in_place(Z, zexp);
#pragma unroll
            for (int nt = 0; nt < KT; ++nt) {
#pragma unroll
                for (int mt = 0; mt < KT; ++mt) Y[nt][mt] = Z[nt][mt];
                yexp[nt] = 0.0;
            }
        } else {
            // Y <- Z with every column renormalised by a power of two
#pragma unroll
            for (int nt = 0; nt < KT; ++nt) {
                double mx = 0.0;
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) mx = fmax(mx, fabs(Z[nt][mt][v]));
                mx = fmax(mx, __shfl_xor(mx, 16, 64));
                mx = fmax(mx, __shfl_xor(mx, 32, 64));
                int ex = 0;
                if (mx > 0.0) (void)frexp(mx, &ex);
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) Y[nt][mt][v] = ldexp(Z[nt][mt][v], -ex);
                yexp[nt] = zexp[nt] + (double)ex;
            }
        }
        if (lane == 0) a.chunk_flags[b * a.C + cc] = did_reset ? 1 : 0;
    }

    store_carry(a.C); // the final state

    // ---- growth of the final state (factorised, not replaced)
    if (a.growth) {
        d4 Z[KT][KT];
#pragma unroll
        for (int nt = 0; nt < KT; ++nt)
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) Z[nt][mt] = Y[nt][mt];
        qr_in_place(Z, yexp);
        if (g == 0) {
#pragma unroll
            for (int nt = 0; nt < KT; ++nt)
                if (16 * nt + c < d) a.growth[b * d + 16 * nt + c] = 0.5 * (log(pprod[nt]) + pexp[nt] * kLn2) * a.growth_scale;
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// The carry kernel for 64 < d <= 128.  A state of 128 x 128 doubles is more than one wave's registers hold, so a
// workgroup of four waves owns a batch item, wave w the columns 32 w .. 32 w + 31 of the state (two panels of
// sixteen).  Z = T_c Y is formed slab by slab from one LDS tile of the chunk product; the factorisation then
// walks the eight panels in order: the wave that owns a panel makes it orthogonal to the finished ones (which
// lie in LDS, in the tile's place), factorises it as above and lays it down for the others.  Arithmetic, layouts
// and bookkeeping are those of the one-wave kernel.
struct WideScratch {
    double rrow[2][16];
    double rperm[2][16];
    double qcol[2][128];
    double diag[128];
    double red[4];
    int hit;
};

// One factorisation of a 128 x 128 matrix held by four waves (wave w: columns 32 w .. 32 w + 31 as two panels) in
// place, Z <- Q: see qr_panels_d.  piv, cexp: pivots and column exponents of this wave's two panels.  Returns the
// largest (squared column norm) / pivot over the whole matrix, the same in every wave.  Finished panels lie in
// LDS at `panels` ([8][128][18] doubles); all four waves must call this together.
__device__ double wide_qr_pass(d4 (&Z)[2][8], double (&piv)[2], double (&cexp)[2], double *panels, WideScratch &s, int wave, int lane)
{
    constexpr int DP = 128, KT = 8, NL = 2, LDQ = 18;
    const int g = lane >> 4, c = lane & 15;
    const int pc = ((c & 3) << 2) | (c >> 2);
    auto panel = [&](int q) { return panels + (size_t)q * DP * LDQ; };
    double norm2[NL];
#pragma unroll
    for (int nl = 0; nl < NL; ++nl) {
        double mx = 0.0;
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) mx = fmax(mx, fabs(Z[nl][mt][v]));
        mx = fmax(mx, __shfl_xor(mx, 16, 64));
        mx = fmax(mx, __shfl_xor(mx, 32, 64));
        int ex = 0;
        if (mx > 0.0) (void)frexp(mx, &ex);
        cexp[nl] = (double)ex;
        double sum = 0.0;
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                Z[nl][mt][v] = ldexp(Z[nl][mt][v], -ex);
                sum = fma(Z[nl][mt][v], Z[nl][mt][v], sum);
            }
        sum += __shfl_xor(sum, 16, 64);
        sum += __shfl_xor(sum, 32, 64);
        norm2[nl] = sum;
        piv[nl] = 1.0;
    }
    __syncthreads(); // (whoever still read the LDS panels or the tile is done)
    // Panel by panel: its owner factorises panel P (by then orthogonal to all finished ones) and lays it down; then
    // every wave makes those of its own panels that come later orthogonal to it, twice in a row (one projection
    // leaves rounding-level remainders of the panel's norm behind), all four waves at work at once.
    auto factor_panel = [&](int P, d4 (&Zp)[KT], double &pv) {
        d4 G = {0., 0., 0., 0.};
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) G = mfma8(Zp[kt][v], Zp[kt][v], G);
        eliminate_panel_d<DP>(G, Zp, pv, s, g, c);
        const double sc = pv > 1.0e-280 ? rsqrt_d(pv) : 0.0;
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) Zp[mt] *= sc;
        if (P + 1 < KT) {
            double *pp = panel(P);
#pragma unroll
            for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                for (int v = 0; v < 4; ++v) pp[(16 * mt + 4 * v + g) * LDQ + pc] = Zp[mt][v];
        }
    };
    auto project_out = [&](int P, d4 (&Zp)[KT]) {
        const double *pq = panel(P);
#pragma unroll 1
        for (int rep = 0; rep < 2; ++rep) {
            d4 R = {0., 0., 0., 0.};
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int v = 0; v < 4; ++v) R = mfma8(pq[(16 * kt + 4 * v + g) * LDQ + pc], Zp[kt][v], R);
            R = -R;
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                const d4 av = *reinterpret_cast<const d4 *>(&pq[(16 * mt + c) * LDQ + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v) Zp[mt] = mfma8(av[v], R[v], Zp[mt]);
            }
        }
    };
#pragma unroll 1
    for (int P = 0; P < KT; ++P) {
        if (wave == P / NL) {
            if (P % NL == 0)
                factor_panel(P, Z[0], piv[0]);
            else
                factor_panel(P, Z[1], piv[1]);
        }
        __syncthreads();
        if (NL * wave > P) project_out(P, Z[0]);
        if (NL * wave + 1 > P) project_out(P, Z[1]);
        // (no barrier: the next panel is written elsewhere, and its owner reads nothing but its own registers before)
    }
    __syncthreads();
    double worst = 1.0;
#pragma unroll
    for (int nl = 0; nl < NL; ++nl) {
        const double ratio = piv[nl] > 1.0e-280 ? norm2[nl] * rcp_d(piv[nl]) : 1.0;
        worst = fmax(worst, ratio);
    }
#pragma unroll
    for (int sft = 1; sft < 16; sft <<= 1) worst = fmax(worst, __shfl_xor(worst, sft, 64));
    if (lane == 0) s.red[wave] = worst;
    __syncthreads();
    worst = fmax(fmax(s.red[0], s.red[1]), fmax(s.red[2], s.red[3]));
    __syncthreads();
    return worst;
}

// Is there a pair of columns of the 128 x 128 matrix Z (held by four waves as in wide_qr_pass) whose squared cosine
// exceeds thr2?  Z goes to LDS panel by panel; every wave takes the pairs whose second column is its own.  The same
// answer in every wave; all four waves must call this together.
__device__ bool wide_colinear(const d4 (&Z)[2][8], double *panels, WideScratch &s, int wave, int lane, int d, double thr2)
{
    constexpr int DP = 128, KT = 8, NL = 2, LDQ = 18;
    const int g = lane >> 4, c = lane & 15;
    const int pc = ((c & 3) << 2) | (c >> 2);
    auto panel = [&](int q) { return panels + (size_t)q * DP * LDQ; };
    __syncthreads(); // the tile, or the panels of a factorisation, are free
#pragma unroll
    for (int nl = 0; nl < NL; ++nl) {
        double *pp = panel(NL * wave + nl);
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) pp[(16 * mt + 4 * v + g) * LDQ + pc] = Z[nl][mt][v];
        d4 Gd = {0., 0., 0., 0.};
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int v = 0; v < 4; ++v) Gd = mfma8(Z[nl][kt][v], Z[nl][kt][v], Gd);
        // G[j][j] for column j = 16 P + c sits in lane (c % 4, c), register c / 4
        double dsel = Gd[0];
        dsel = (c >> 2) == 1 ? Gd[1] : dsel;
        dsel = (c >> 2) == 2 ? Gd[2] : dsel;
        dsel = (c >> 2) == 3 ? Gd[3] : dsel;
        if (g == (c & 3)) s.diag[32 * wave + 16 * nl + c] = dsel;
    }
    if (threadIdx.x == 0) s.hit = 0;
    __syncthreads();
    bool hit = false;
#pragma unroll
    for (int nl = 0; nl < NL; ++nl) {
        const int P = NL * wave + nl;
        const double dc = s.diag[16 * P + c];
        for (int q = 0; q <= P; ++q) {
            const double *pq = panel(q);
            d4 Gt = {0., 0., 0., 0.}; // rows: columns 16 q + .. of Z, columns: 16 P + c
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int v = 0; v < 4; ++v) Gt = mfma8(pq[(16 * kt + 4 * v + g) * LDQ + pc], Z[nl][kt][v], Gt);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * q + 4 * v + g, col = 16 * P + c;
                const double dr = s.diag[row];
                const double x = Gt[v];
                if (row < col && col < d && x * x > thr2 * dr * dc) hit = true;
            }
        }
    }
    if (__builtin_amdgcn_ballot_w64(hit) != 0 && lane == 0) s.hit = 1;
    __syncthreads();
    return s.hit != 0;
}

template <typename IO> __global__ __launch_bounds__(256) void reset_carry_wide_kernel(ResetArgs a)
{
    constexpr int DP = 128, KT = DP / 16, NL = 2, NW = 4, LDT = DP + 2, LDQ = 18;
    constexpr int TQ = DP * DP / 4 / (NW * 64); // 32-byte pieces of the chunk product per thread
    extern __shared__ __align__(32) unsigned char smem[];
    double *tile = reinterpret_cast<double *>(smem); // [128][130]: chunk product, columns in perm16 order
    auto panel = [&](int q) { return reinterpret_cast<double *>(smem) + (size_t)q * DP * LDQ; }; // [8][128][18], after the product
    WideScratch &s = *reinterpret_cast<WideScratch *>(smem + (size_t)KT * DP * LDQ * sizeof(double));
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const int pc = ((c & 3) << 2) | (c >> 2); // position of column c inside a stored panel
    const int d = a.d;
    const long long b = blockIdx.x;
    const size_t tot_mant = (size_t)DP * a.tot_cols * sizeof(double);
    const size_t car_mant = (size_t)DP * a.car_cols * sizeof(double);

    d4 Y[NL][KT]; // Y[nl][mt][v] = entry (row 16 mt + 4 v + g, column 32 wave + 16 nl + c), columns scaled by 2^yexp
    double yexp[NL], pprod[NL], pexp[NL];
#pragma unroll
    for (int nl = 0; nl < NL; ++nl) {
        yexp[nl] = 0.0;
        pprod[nl] = 1.0;
        pexp[nl] = 0.0;
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) Y[nl][mt][v] = (16 * mt + 4 * v + g == 32 * wave + 16 * nl + c) ? 1.0 : 0.0;
    }
    if (a.s0) {
        const IO *gp = reinterpret_cast<const IO *>(a.s0) + (size_t)b * d * d * 2;
#pragma unroll
        for (int nl = 0; nl < NL; ++nl) {
            const int col = 32 * wave + 16 * nl + c;
            if (col < d) {
                double cmax = -__builtin_huge_val();
                for (int i = 0; i < d; ++i) cmax = fmax(cmax, (double)gp[((size_t)i * d + col) * 2]);
                yexp[nl] = cmax > -__builtin_huge_val() ? ceil(cmax * kLog2e) : 0.0;
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = 16 * mt + 4 * v + g;
                        double val = 0.0;
                        if (row < d) {
                            const IO *e = gp + ((size_t)row * d + col) * 2;
                            const double t = (double)e[0] * kLog2e - yexp[nl];
                            val = t > -1000.0 ? exp2(t) : 0.0;
                            if ((int)rint((double)e[1] * 0.318309886183790671538) & 1) val = -val;
                        }
                        Y[nl][mt][v] = val;
                    }
            }
        }
    }

    auto store_carry = [&](long long cc) {
        unsigned char *dst = a.carries + (b * (a.C + 1) + cc) * a.car_stride;
        double *mp = reinterpret_cast<double *>(dst);
        double *ep = reinterpret_cast<double *>(dst + car_mant);
#pragma unroll
        for (int nl = 0; nl < NL; ++nl) {
            const int col = 32 * wave + 16 * nl + c;
            if (col < a.car_cols) {
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int row = 16 * mt + 4 * v + g;
                        mp[(size_t)row * a.car_cols + col] = (row < d && col < d) ? Y[nl][mt][v] : 0.0;
                    }
                if (g == 0) ep[col] = col < d ? yexp[nl] : 0.0;
            }
        }
    };

    auto qr_pass = [&](d4 (&Z)[NL][KT], double (&piv)[NL], double (&cexp)[NL]) { return wide_qr_pass(Z, piv, cexp, panel(0), s, wave, lane); };
    auto qr_in_place = [&](d4 (&Z)[NL][KT], const double (&colexp)[NL]) {
        double piv[NL], piv2[NL], ce[NL], ce2[NL];
        const double amp = qr_pass(Z, piv, ce);
#pragma unroll
        for (int nl = 0; nl < NL; ++nl) {
            piv2[nl] = 1.0;
            ce2[nl] = 0.0;
        }
        if (amp > (sizeof(IO) == 4 ? 1.0e10 : 1.0e3)) (void)qr_pass(Z, piv2, ce2); // (the same in every wave)
#pragma unroll
        for (int nl = 0; nl < NL; ++nl)
            if (piv[nl] > 1.0e-280 && piv2[nl] > 1.0e-280) {
                int e;
                pprod[nl] = frexp(pprod[nl] * piv[nl] * piv2[nl], &e);
                pexp[nl] += 2.0 * (colexp[nl] + ce[nl] + ce2[nl]) + (double)e;
            }
    };

    for (long long cc = 0; cc < a.C; ++cc) {
        store_carry(cc);
        const unsigned char *tp = a.totals + (b * a.C + cc) * a.tot_stride;
        const double tex = *reinterpret_cast<const double *>(tp + tot_mant);
        __syncthreads(); // (the panels of the chunk before are done with)
#pragma unroll 4
        for (int q = 0; q < TQ; ++q) {
            const int piece = tid + NW * 64 * q;
            const int row = piece / (DP / 4), c4 = 4 * (piece % (DP / 4));
            const int p4 = (c4 & ~15) | ((c4 >> 2) & 3);
            d4 val = {0., 0., 0., 0.};
            if (c4 < a.tot_cols) val = *reinterpret_cast<const d4 *>(reinterpret_cast<const double *>(tp) + (size_t)row * a.tot_cols + c4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                double x = val[e];
                if (row >= d || c4 + e >= d) x = (c4 + e == row) ? 1.0 : 0.0; // identity block past d
                tile[row * LDT + p4 + 4 * e] = x;
            }
        }
        __syncthreads();
        // ---- Z = T_c Y
        d4 Z[NL][KT];
#pragma unroll
        for (int nl = 0; nl < NL; ++nl)
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) Z[nl][mt] = d4{0., 0., 0., 0.};
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) {
                const d4 av = *reinterpret_cast<const d4 *>(&tile[(16 * mt + c) * LDT + 16 * kt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v)
#pragma unroll
                    for (int nl = 0; nl < NL; ++nl) Z[nl][mt] = mfma8(av[v], Y[nl][kt][v], Z[nl][mt]);
            }
        double zexp[NL];
#pragma unroll
        for (int nl = 0; nl < NL; ++nl) zexp[nl] = yexp[nl] + tex;

        const long long t_end = (cc + 1) * a.L;
        const bool boundary = t_end <= a.T && a.policy >= 0;
        bool did_reset = false;
        if (boundary) {
            did_reset = a.policy == 1;
            if (!did_reset) {
                did_reset = wide_colinear(Z, panel(0), s, wave, lane, d, (double)a.cos_threshold * (double)a.cos_threshold);
            }
        }
        if (did_reset) {
            qr_in_place(Z, zexp);
#pragma unroll
            for (int nl = 0; nl < NL; ++nl) {
#pragma unroll
                for (int mt = 0; mt < KT; ++mt) Y[nl][mt] = Z[nl][mt];
                yexp[nl] = 0.0;
            }
        } else {
#pragma unroll
            for (int nl = 0; nl < NL; ++nl) {
                double mx = 0.0;
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) mx = fmax(mx, fabs(Z[nl][mt][v]));
                mx = fmax(mx, __shfl_xor(mx, 16, 64));
                mx = fmax(mx, __shfl_xor(mx, 32, 64));
                int ex = 0;
                if (mx > 0.0) (void)frexp(mx, &ex);
#pragma unroll
                for (int mt = 0; mt < KT; ++mt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) Y[nl][mt][v] = ldexp(Z[nl][mt][v], -ex);
                yexp[nl] = zexp[nl] + (double)ex;
            }
        }
        if (tid == 0) a.chunk_flags[b * a.C + cc] = did_reset ? 1 : 0;
    }

    store_carry(a.C); // the final state

    if (a.growth) { // growth of the final state (factorised, not replaced)
        d4 Z[NL][KT];
#pragma unroll
        for (int nl = 0; nl < NL; ++nl)
#pragma unroll
            for (int mt = 0; mt < KT; ++mt) Z[nl][mt] = Y[nl][mt];
        qr_in_place(Z, yexp);
        if (g == 0) {
#pragma unroll
            for (int nl = 0; nl < NL; ++nl) {
                const int col = 32 * wave + 16 * nl + c;
                if (col < d) a.growth[b * d + col] = 0.5 * (log(pprod[nl]) + pexp[nl] * kLn2) * a.growth_scale;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// The selective-resetting scan in the order of the paper's own parallel prefix scan (Section 5, eq. 28;
// Appendix C).  Elements (X_0, A_1, ..., A_T) are GOOM matrices; parallel step k works on blocks of 2^k
// elements, updating every element of a block's upper half from the last element of its lower half.  With all
// bias slots zero at the start every tuple (A*, B*) has one non-zero slot, so an element is one matrix M and a
// flag "has been reset" (the bias slot is the occupied one): a flagged element ignores what precedes it
// (A* = 0), an unflagged one becomes LMME(M_curr, M_prev) and inherits the flag of prev.  Before each parallel
// step every unflagged element that S selects is replaced by R(M) and flagged (tree_reset_kernel); the
// products of a step are batched LMMEs of the chain kernel, scattered back by tree_scatter_kernel.
struct TreeResetArgs {
    void *M;             // [n][d][d] GOOMs of one batch item, n = T + 1 elements
    unsigned char *flag; // [n]
    long long n;
    int d;
    int policy;
    float cos_threshold;
};

template <int DP, typename IO> __global__ __launch_bounds__(64) void tree_reset_kernel(TreeResetArgs a)
{
    constexpr int KT = DP / 16;
    __shared__ __align__(32) WaveD<DP> s;
    const int lane = threadIdx.x;
    const int g = lane >> 4, c = lane & 15;
    const int d = a.d;
    const long long i = blockIdx.x;
    if (a.flag[i] || a.policy < 0) return; // whole wave
    IO *mp = static_cast<IO *>(a.M) + (size_t)i * d * d * 2;
    // columns scaled to a largest entry of 1 (identity block past d)
    d4 Z[KT][KT];
    bool any = false;
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) {
        const int col = 16 * nt + c;
        double re[KT][4], im[KT][4];
        double cmax = -__builtin_huge_val();
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * mt + 4 * v + g;
                double r = row == col ? 0.0 : -__builtin_huge_val(), im_ = 0.0;
                if (row < d && col < d) {
                    r = (double)mp[((size_t)row * d + col) * 2];
                    im_ = (double)mp[((size_t)row * d + col) * 2 + 1];
                    any = any || r > -__builtin_huge_val();
                }
                re[mt][v] = r;
                im[mt][v] = im_;
                cmax = fmax(cmax, r);
            }
        cmax = fmax(cmax, __shfl_xor(cmax, 16, 64));
        cmax = fmax(cmax, __shfl_xor(cmax, 32, 64));
        const bool zero_col = !(cmax > -__builtin_huge_val());
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                double x = zero_col ? 0.0 : exp(re[mt][v] - cmax);
                if ((int)rint(im[mt][v] * 0.318309886183790671538) & 1) x = -x;
                Z[nt][mt][v] = x;
            }
    }
    if (__builtin_amdgcn_ballot_w64(any) == 0) return; // a zero matrix is never selected
    bool sel = a.policy == 1;
    if (!sel) {
        // squared cosines between columns, tile by tile of the Gram matrix
#pragma unroll
        for (int nt = 0; nt < KT; ++nt) {
            d4 Gd = {0., 0., 0., 0.};
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int v = 0; v < 4; ++v) Gd = mfma8(Z[nt][kt][v], Z[nt][kt][v], Gd);
            double dsel = Gd[0];
            dsel = (c >> 2) == 1 ? Gd[1] : dsel;
            dsel = (c >> 2) == 2 ? Gd[2] : dsel;
            dsel = (c >> 2) == 3 ? Gd[3] : dsel;
            if (g == (c & 3)) s.diag[16 * nt + c] = dsel;
        }
        wave_sync();
        bool hit = false;
        const double thr2 = (double)a.cos_threshold * (double)a.cos_threshold;
#pragma unroll
        for (int nt = 0; nt < KT; ++nt) {
            const double dc = s.diag[16 * nt + c];
#pragma unroll
            for (int mt = 0; mt <= nt; ++mt) {
                d4 Gt = {0., 0., 0., 0.};
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) Gt = mfma8(Z[mt][kt][v], Z[nt][kt][v], Gt);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = 16 * mt + 4 * v + g, col = 16 * nt + c;
                    const double dr = s.diag[row];
                    if (row < col && col < d && Gt[v] * Gt[v] > thr2 * dr * dc) hit = true;
                }
            }
        }
        wave_sync();
        sel = __builtin_amdgcn_ballot_w64(hit) != 0;
    }
    if (!sel) return;
    double piv[KT], ce[KT];
    const double amp = qr_panels_d<DP>(Z, piv, ce, s, g, c);
    if (amp > (sizeof(IO) == 4 ? 1.0e10 : 1.0e3)) (void)qr_panels_d<DP>(Z, piv, ce, s, g, c);
    const IO pi = sizeof(IO) == 4 ? (IO)3.14159274101257324219f : (IO)3.14159265358979311600;
#pragma unroll
    for (int nt = 0; nt < KT; ++nt)
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * mt + 4 * v + g, col = 16 * nt + c;
                if (row < d && col < d) {
                    const double q = Z[nt][mt][v];
                    mp[((size_t)row * d + col) * 2] = (IO)(q != 0.0 ? log(fabs(q)) : -__builtin_huge_val());
                    mp[((size_t)row * d + col) * 2 + 1] = q < 0.0 ? pi : (IO)0;
                }
            }
    if (lane == 0) a.flag[i] = 1;
}

// The same for 64 < d <= 128: four waves per element, the factorisation and the cosine test of the wide carry kernel.
template <typename IO> __global__ __launch_bounds__(256) void tree_reset_wide_kernel(TreeResetArgs a)
{
    constexpr int DP = 128, KT = 8, NL = 2, LDQ = 18;
    extern __shared__ __align__(32) unsigned char smem[];
    double *panels = reinterpret_cast<double *>(smem);
    WideScratch &s = *reinterpret_cast<WideScratch *>(smem + (size_t)KT * DP * LDQ * sizeof(double));
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const int d = a.d;
    const long long i = blockIdx.x;
    if (a.flag[i] || a.policy < 0) return; // whole workgroup
    IO *mp = static_cast<IO *>(a.M) + (size_t)i * d * d * 2;
    d4 Z[NL][KT];
    bool any = false;
#pragma unroll
    for (int nl = 0; nl < NL; ++nl) {
        const int col = 32 * wave + 16 * nl + c;
        double cmax = -__builtin_huge_val();
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * mt + 4 * v + g;
                double r = row == col ? 0.0 : -__builtin_huge_val();
                if (row < d && col < d) {
                    r = (double)mp[((size_t)row * d + col) * 2];
                    any = any || r > -__builtin_huge_val();
                }
                Z[nl][mt][v] = r;
                cmax = fmax(cmax, r);
            }
        cmax = fmax(cmax, __shfl_xor(cmax, 16, 64));
        cmax = fmax(cmax, __shfl_xor(cmax, 32, 64));
        const bool zero_col = !(cmax > -__builtin_huge_val());
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * mt + 4 * v + g;
                double x = zero_col ? 0.0 : exp(Z[nl][mt][v] - cmax);
                if (row < d && col < d && ((int)rint((double)mp[((size_t)row * d + col) * 2 + 1] * 0.318309886183790671538) & 1)) x = -x;
                Z[nl][mt][v] = x;
            }
    }
    if (tid == 0) s.hit = 0;
    __syncthreads();
    if (__builtin_amdgcn_ballot_w64(any) != 0 && lane == 0) s.hit = 1;
    __syncthreads();
    if (s.hit == 0) return; // a zero matrix is never selected (the same in every wave)
    bool sel = a.policy == 1;
    if (!sel) sel = wide_colinear(Z, panels, s, wave, lane, d, (double)a.cos_threshold * (double)a.cos_threshold);
    if (!sel) return;
    double piv[NL], ce[NL];
    const double amp = wide_qr_pass(Z, piv, ce, panels, s, wave, lane);
    if (amp > (sizeof(IO) == 4 ? 1.0e10 : 1.0e3)) (void)wide_qr_pass(Z, piv, ce, panels, s, wave, lane);
    const IO pi = sizeof(IO) == 4 ? (IO)3.14159274101257324219f : (IO)3.14159265358979311600;
#pragma unroll
    for (int nl = 0; nl < NL; ++nl)
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * mt + 4 * v + g, col = 32 * wave + 16 * nl + c;
                if (row < d && col < d) {
                    const double q = Z[nl][mt][v];
                    mp[((size_t)row * d + col) * 2] = (IO)(q != 0.0 ? log(fabs(q)) : -__builtin_huge_val());
                    mp[((size_t)row * d + col) * 2 + 1] = q < 0.0 ? pi : (IO)0;
                }
            }
    if (tid == 0) a.flag[i] = 1;
}

// After the products of a parallel step: element i = block * 2 half + half + u takes tmp[block][u] unless it is
// flagged, and inherits the flag of j = block * 2 half + half - 1.  One workgroup per element.
template <typename IO> __global__ __launch_bounds__(256) void tree_scatter_kernel(IO *M, const IO *tmp, unsigned char *flag, long long n, int d,
                                                                                  long long half)
{
    const long long e = blockIdx.x; // index among the updated elements, block by block
    const long long block = e / half, u = e % half;
    const long long i = block * 2 * half + half + u, j = block * 2 * half + half - 1;
    if (i >= n) return;
    const unsigned char fi = flag[i], fj = flag[j];
    __syncthreads();
    if (!fi) {
        const size_t nn = (size_t)d * d * 2;
        for (size_t q = threadIdx.x; q < nn; q += 256) M[(size_t)i * nn + q] = tmp[(size_t)e * nn + q];
        if (threadIdx.x == 0) flag[i] = fj;
    }
}

// elements of one batch item: X_0 (given, or the identity) and the T matrices; flags cleared
template <typename IO> __global__ __launch_bounds__(256) void tree_init_kernel(const IO *J, const IO *S0, IO *M, unsigned char *flag, long long n, int d)
{
    const long long i = blockIdx.x;
    const size_t nn = (size_t)d * d * 2;
    const IO ninf = sizeof(IO) == 4 ? (IO)-__builtin_huge_valf() : (IO)-__builtin_huge_val();
    for (size_t q = threadIdx.x; q < nn; q += 256) {
        IO v;
        if (i > 0) v = J[(size_t)(i - 1) * nn + q];
        else if (S0) v = S0[q];
        else v = (q & 1) ? (IO)0 : (((q / 2) / d == (q / 2) % d) ? (IO)0 : ninf);
        M[(size_t)i * nn + q] = v;
    }
    if (threadIdx.x == 0) flag[i] = 0;
}

template <typename IO> __global__ __launch_bounds__(256) void tree_finish_kernel(const IO *M, const unsigned char *flag, IO *states, unsigned char *out_flags,
                                                                                 long long n, int d)
{
    const long long t = blockIdx.x; // state after step t + 1 = element t + 1
    const size_t nn = (size_t)d * d * 2;
    for (size_t q = threadIdx.x; q < nn; q += 256) states[(size_t)t * nn + q] = M[(size_t)(t + 1) * nn + q];
    if (out_flags && threadIdx.x == 0) out_flags[t] = flag[t + 1];
}

// Spectrum from the input states (paper Section 4.2.1, groups (b)-(d)): one wave per step t.
// The input state S_{t-1} is log-scaled column by column and exponentiated, its QR gives the
// orthonormal basis Q_{t-1}; J_t (scaled by one power of two for the whole matrix) is applied to
// it on the matrix unit, and the QR of the result gives R_t; log R_kk goes to steplog[b][t][k].
// Every step is independent of the others.
struct StepArgs {
    const float *J;      // [batch][T][d][d] GOOMs
    const float *S0;     // NULL (identity) or [batch][d][d] GOOMs
    const float *states; // [batch][T][d][d] GOOMs: entry t holds the state after step t + 1
    double *steplog;     // [batch][T][d]
    long long T;
    int d;
};

template <int DP> __global__ __launch_bounds__(64) void lyap_step_kernel(StepArgs a)
{
    constexpr int KT = DP / 16;
    constexpr int LDT = DP + 4;
    constexpr int TQ = DP * DP / 4 / 64;
    __shared__ __align__(16) Wave<DP> s;
    const int lane = threadIdx.x;
    const int g = lane >> 4, c = lane & 15;
    const int d = a.d;
    const long long b = blockIdx.x / a.T, t = blockIdx.x % a.T;
    const float kLog2eF = 1.44269504088896340736f;

    // ---- input state, columns scaled to largest entry 1 (identity block past d)
    const float *src = t == 0 ? (a.S0 ? a.S0 + (size_t)b * d * d * 2 : nullptr) : a.states + (size_t)(b * a.T + t - 1) * d * d * 2;
    f4 Q[KT][KT];
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) {
        const int col = 16 * nt + c;
        float re[KT][4], im[KT][4];
        float cmax = -__builtin_huge_valf();
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * mt + 4 * g + v;
                float r = row == col ? 0.0f : -__builtin_huge_valf(), i = 0.0f;
                if (src && row < d && col < d) {
                    const float2 e = *reinterpret_cast<const float2 *>(src + ((size_t)row * d + col) * 2);
                    r = e.x;
                    i = e.y;
                }
                re[mt][v] = r;
                im[mt][v] = i;
                cmax = fmaxf(cmax, r);
            }
        cmax = fmaxf(cmax, __shfl_xor(cmax, 16, 64));
        cmax = fmaxf(cmax, __shfl_xor(cmax, 32, 64));
        const bool zero_col = !(cmax > -__builtin_huge_valf());
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float x = zero_col ? 0.0f : __builtin_amdgcn_exp2f((re[mt][v] - cmax) * kLog2eF);
                if ((int)rintf(im[mt][v] * 0.318309886183790671538f) & 1) x = -x;
                Q[nt][mt][v] = x;
            }
    }
    {
        double piv[KT];
        const float amp = qr_panels<DP>(Q, piv, s, g, c);
        if (amp > 65536.0f) (void)qr_panels<DP>(Q, piv, s, g, c);
    }

    // ---- J_t as reals scaled by 2^-sh, sh from the largest entry; identity block past d
    const float *jp = a.J + (size_t)(b * a.T + t) * d * d * 2;
    float jre[TQ][4], jim[TQ][4];
    float jmax = -__builtin_huge_valf();
#pragma unroll
    for (int q = 0; q < TQ; ++q) {
        const int piece = lane + 64 * q;
        const int row = piece / (DP / 4), c4 = 4 * (piece % (DP / 4));
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float r = -__builtin_huge_valf(), i = 0.0f;
            if (row < d && c4 + e < d) {
                const float2 v = *reinterpret_cast<const float2 *>(jp + ((size_t)row * d + c4 + e) * 2);
                r = v.x;
                i = v.y;
            }
            jre[q][e] = r;
            jim[q][e] = i;
            jmax = fmaxf(jmax, r);
        }
    }
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) jmax = fmaxf(jmax, __shfl_xor(jmax, sft, 64));
    const float sh = jmax > -__builtin_huge_valf() ? ceilf(jmax * kLog2eF) : 0.0f;
#pragma unroll
    for (int q = 0; q < TQ; ++q) {
        const int piece = lane + 64 * q;
        const int row = piece / (DP / 4), c4 = 4 * (piece % (DP / 4));
        f4 val;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float x = __builtin_amdgcn_exp2f(__builtin_fmaf(jre[q][e], kLog2eF, -sh));
            if ((int)rintf(jim[q][e] * 0.318309886183790671538f) & 1) x = -x;
            if (row >= d || c4 + e >= d) x = (c4 + e == row) ? 1.0f : 0.0f;
            val[e] = x;
        }
        *reinterpret_cast<f4 *>(&s.tile[row * LDT + c4]) = val;
    }
    wave_sync();
    f4 Z[KT][KT];
#pragma unroll
    for (int nt = 0; nt < KT; ++nt)
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) Z[nt][mt] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) {
            const f4 av = *reinterpret_cast<const f4 *>(&s.tile[(16 * mt + c) * LDT + 16 * kt + 4 * g]);
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int nt = 0; nt < KT; ++nt) Z[nt][mt] = mfma4(av[v], Q[nt][kt][v], Z[nt][mt]);
        }
    wave_sync();
    double piv[KT], piv2[KT];
    const float amp = qr_panels<DP>(Z, piv, s, g, c);
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) piv2[nt] = 1.0;
    if (amp > 65536.0f) (void)qr_panels<DP>(Z, piv2, s, g, c);
    if (g == 0) {
#pragma unroll
        for (int nt = 0; nt < KT; ++nt) {
            const int col = 16 * nt + c;
            if (col < d) {
                const double p = piv[nt] * piv2[nt];
                a.steplog[(size_t)(b * a.T + t) * d + col] = p > 1.0e-60 ? 0.5 * log(p) + (double)sh * kLn2 : -__builtin_huge_val();
            }
        }
    }
}

// The same for complex128 GOOMs, in double throughout: the factorisations and the product run on the double matrix
// instruction in the layout of the carry kernel above (register v of lane (g, c) holds row 4 v + g; whatever is read
// from LDS as a four-vector stores index 4 v + g at position 4 g + v).
struct StepArgsD {
    const double *J, *S0, *states;
    double *steplog;
    long long T;
    int d;
};

template <int DP> __global__ __launch_bounds__(64) void lyap_step_kernel_d(StepArgsD a)
{
    constexpr int KT = DP / 16;
    constexpr int LDT = WaveD<DP>::LDT;
    constexpr int TQ = DP * DP / 4 / 64;
    __shared__ __align__(32) WaveD<DP> s;
    const int lane = threadIdx.x;
    const int g = lane >> 4, c = lane & 15;
    const int d = a.d;
    const long long b = blockIdx.x / a.T, t = blockIdx.x % a.T;
    auto is_odd = [](double im) { return ((int)rint(im * 0.318309886183790671538) & 1) != 0; };

    // ---- input state, columns scaled to largest entry 1 (identity block past d)
    const double *src = t == 0 ? (a.S0 ? a.S0 + (size_t)b * d * d * 2 : nullptr) : a.states + (size_t)(b * a.T + t - 1) * d * d * 2;
    d4 Q[KT][KT];
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) {
        const int col = 16 * nt + c;
        double cmax = -__builtin_huge_val();
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * mt + 4 * v + g;
                double r = row == col ? 0.0 : -__builtin_huge_val();
                if (src && row < d && col < d) r = src[((size_t)row * d + col) * 2];
                Q[nt][mt][v] = r;
                cmax = fmax(cmax, r);
            }
        cmax = fmax(cmax, __shfl_xor(cmax, 16, 64));
        cmax = fmax(cmax, __shfl_xor(cmax, 32, 64));
        const bool zero_col = !(cmax > -__builtin_huge_val());
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * mt + 4 * v + g;
                const double tt = (Q[nt][mt][v] - cmax) * kLog2e;
                double x = (zero_col || !(tt > -1000.0)) ? 0.0 : exp2(tt);
                if (src && row < d && col < d && is_odd(src[((size_t)row * d + col) * 2 + 1])) x = -x;
                Q[nt][mt][v] = x;
            }
    }
    {
        double piv[KT], ce[KT];
        const double amp = qr_panels_d<DP>(Q, piv, ce, s, g, c);
        if (amp > 1.0e3) (void)qr_panels_d<DP>(Q, piv, ce, s, g, c);
    }

    // ---- J_t as reals scaled by 2^-sh, sh from the largest entry; identity block past d
    const double *jp = a.J + (size_t)(b * a.T + t) * d * d * 2;
    double jmax = -__builtin_huge_val();
    for (int q = 0; q < TQ; ++q) {
        const int piece = lane + 64 * q;
        const int row = piece / (DP / 4), c4 = 4 * (piece % (DP / 4));
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (row < d && c4 + e < d) jmax = fmax(jmax, jp[((size_t)row * d + c4 + e) * 2]);
    }
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) jmax = fmax(jmax, __shfl_xor(jmax, sft, 64));
    const double sh = jmax > -__builtin_huge_val() ? ceil(jmax * kLog2e) : 0.0;
    for (int q = 0; q < TQ; ++q) {
        const int piece = lane + 64 * q;
        const int row = piece / (DP / 4), c4 = 4 * (piece % (DP / 4));
        const int p4 = (c4 & ~15) | ((c4 >> 2) & 3);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            double x = (c4 + e == row) ? 1.0 : 0.0;
            if (row < d && c4 + e < d) {
                const double *v = jp + ((size_t)row * d + c4 + e) * 2;
                const double tt = __builtin_fma(v[0], kLog2e, -sh);
                x = tt > -1000.0 ? exp2(tt) : 0.0;
                if (is_odd(v[1])) x = -x;
            }
            s.tile[row * LDT + p4 + 4 * e] = x;
        }
    }
    wave_sync();
    d4 Z[KT][KT];
#pragma unroll
    for (int nt = 0; nt < KT; ++nt)
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) Z[nt][mt] = d4{0., 0., 0., 0.};
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) {
            const d4 av = *reinterpret_cast<const d4 *>(&s.tile[(16 * mt + c) * LDT + 16 * kt + 4 * g]);
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int nt = 0; nt < KT; ++nt) Z[nt][mt] = mfma8(av[v], Q[nt][kt][v], Z[nt][mt]);
        }
    wave_sync();
    double piv[KT], piv2[KT], ce[KT], ce2[KT];
    const double amp = qr_panels_d<DP>(Z, piv, ce, s, g, c);
#pragma unroll
    for (int nt = 0; nt < KT; ++nt) {
        piv2[nt] = 1.0;
        ce2[nt] = 0.0;
    }
    if (amp > 1.0e3) (void)qr_panels_d<DP>(Z, piv2, ce2, s, g, c);
    if (g == 0) {
#pragma unroll
        for (int nt = 0; nt < KT; ++nt) {
            const int col = 16 * nt + c;
            if (col < d) {
                const bool ok = piv[nt] > 1.0e-280 && piv2[nt] > 1.0e-280;
                a.steplog[(size_t)(b * a.T + t) * d + col] =
                    ok ? 0.5 * (log(piv[nt]) + log(piv2[nt])) + (ce[nt] + ce2[nt] + sh) * kLn2 : -__builtin_huge_val();
            }
        }
    }
}

// The per-step estimator for 64 < d <= 128: a workgroup of four waves per step, the state's columns divided among
// them as in reset_carry_wide_kernel, everything in double for both formats.
template <typename IO> __global__ __launch_bounds__(256) void lyap_step_wide_kernel(const IO *J, const IO *S0, const IO *states, double *steplog,
                                                                                    long long T, int d)
{
    constexpr int DP = 128, KT = 8, NL = 2, NW = 4, LDT = DP + 2, LDQ = 18;
    constexpr int TQ = DP * DP / 4 / (NW * 64);
    extern __shared__ __align__(32) unsigned char smem[];
    double *tile = reinterpret_cast<double *>(smem);
    double *panels = reinterpret_cast<double *>(smem);
    WideScratch &s = *reinterpret_cast<WideScratch *>(smem + (size_t)KT * DP * LDQ * sizeof(double));
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const long long b = blockIdx.x / T, t = blockIdx.x % T;
    auto is_odd = [](double im) { return ((int)rint(im * 0.318309886183790671538) & 1) != 0; };

    // ---- input state, columns scaled to largest entry 1 (identity block past d), then its orthonormal factor
    const IO *src = t == 0 ? (S0 ? S0 + (size_t)b * d * d * 2 : nullptr) : states + (size_t)(b * T + t - 1) * d * d * 2;
    d4 Q[NL][KT];
#pragma unroll
    for (int nl = 0; nl < NL; ++nl) {
        const int col = 32 * wave + 16 * nl + c;
        double cmax = -__builtin_huge_val();
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * mt + 4 * v + g;
                double r = row == col ? 0.0 : -__builtin_huge_val();
                if (src && row < d && col < d) r = (double)src[((size_t)row * d + col) * 2];
                Q[nl][mt][v] = r;
                cmax = fmax(cmax, r);
            }
        cmax = fmax(cmax, __shfl_xor(cmax, 16, 64));
        cmax = fmax(cmax, __shfl_xor(cmax, 32, 64));
        const bool zero_col = !(cmax > -__builtin_huge_val());
#pragma unroll
        for (int mt = 0; mt < KT; ++mt)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = 16 * mt + 4 * v + g;
                const double tt = (Q[nl][mt][v] - cmax) * kLog2e;
                double x = (zero_col || !(tt > -1000.0)) ? 0.0 : exp2(tt);
                if (src && row < d && col < d && is_odd((double)src[((size_t)row * d + col) * 2 + 1])) x = -x;
                Q[nl][mt][v] = x;
            }
    }
    {
        double piv[NL], ce[NL];
        const double amp = wide_qr_pass(Q, piv, ce, panels, s, wave, lane);
        if (amp > 1.0e3) (void)wide_qr_pass(Q, piv, ce, panels, s, wave, lane);
    }

    // ---- J_t as reals scaled by 2^-sh, sh from the largest entry; identity block past d
    const IO *jp = J + (size_t)(b * T + t) * d * d * 2;
    double jmax = -__builtin_huge_val();
    for (int e = tid; e < d * d; e += NW * 64) jmax = fmax(jmax, (double)jp[(size_t)e * 2]);
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) jmax = fmax(jmax, __shfl_xor(jmax, sft, 64));
    __syncthreads(); // (the panels of the factorisation above are done with; s.red is free)
    if (lane == 0) s.red[wave] = jmax;
    __syncthreads();
    jmax = fmax(fmax(s.red[0], s.red[1]), fmax(s.red[2], s.red[3]));
    const double sh = jmax > -__builtin_huge_val() ? ceil(jmax * kLog2e) : 0.0;
    for (int q = 0; q < TQ; ++q) {
        const int piece = tid + NW * 64 * q;
        const int row = piece / (DP / 4), c4 = 4 * (piece % (DP / 4));
        const int p4 = (c4 & ~15) | ((c4 >> 2) & 3);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            double x = (c4 + e == row) ? 1.0 : 0.0;
            if (row < d && c4 + e < d) {
                const IO *v = jp + ((size_t)row * d + c4 + e) * 2;
                const double tt = __builtin_fma((double)v[0], kLog2e, -sh);
                x = tt > -1000.0 ? exp2(tt) : 0.0;
                if (is_odd((double)v[1])) x = -x;
            }
            tile[row * LDT + p4 + 4 * e] = x;
        }
    }
    __syncthreads();
    d4 Z[NL][KT];
#pragma unroll
    for (int nl = 0; nl < NL; ++nl)
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) Z[nl][mt] = d4{0., 0., 0., 0.};
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int mt = 0; mt < KT; ++mt) {
            const d4 av = *reinterpret_cast<const d4 *>(&tile[(16 * mt + c) * LDT + 16 * kt + 4 * g]);
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int nl = 0; nl < NL; ++nl) Z[nl][mt] = mfma8(av[v], Q[nl][kt][v], Z[nl][mt]);
        }
    double piv[NL], piv2[NL], ce[NL], ce2[NL];
    const double amp = wide_qr_pass(Z, piv, ce, panels, s, wave, lane); // (its first barrier comes after the reads of the tile)
#pragma unroll
    for (int nl = 0; nl < NL; ++nl) {
        piv2[nl] = 1.0;
        ce2[nl] = 0.0;
    }
    if (amp > 1.0e3) (void)wide_qr_pass(Z, piv2, ce2, panels, s, wave, lane);
    if (g == 0) {
#pragma unroll
        for (int nl = 0; nl < NL; ++nl) {
            const int col = 32 * wave + 16 * nl + c;
            if (col < d) {
                const bool ok = piv[nl] > 1.0e-280 && piv2[nl] > 1.0e-280;
                steplog[(size_t)(b * T + t) * d + col] = ok ? 0.5 * (log(piv[nl]) + log(piv2[nl])) + (ce[nl] + ce2[nl] + sh) * kLn2 : -__builtin_huge_val();
            }
        }
    }
}

// lambda[b][k] = scale * sum_t steplog[b][t][k], summed in a fixed order: kSlices slices of the
// steps per batch item, partial sums in the workspace, then one block adds the slices.
constexpr int kSlices = 64;

__global__ __launch_bounds__(256) void steplog_partial_kernel(const double *steplog, double *partial, long long T, int d)
{
    __shared__ double red[256];
    const long long b = blockIdx.x / kSlices;
    const int slice = blockIdx.x % kSlices;
    const int r = threadIdx.x >> 6; // 4 groups of 64 threads; thread k < d of a group owns exponent k (and k + 64 above 64)
    const long long per = (T + kSlices - 1) / kSlices;
    const long long lo = slice * per, hi = lo + per < T ? lo + per : T;
    for (int k0 = 0; k0 < d; k0 += 64) { // (the same trips for every thread: there are barriers inside)
        const int kk = threadIdx.x & 63, k = k0 + kk;
        double acc = 0.0;
        if (k < d)
            for (long long t = lo + r; t < hi; t += 4) acc += steplog[(size_t)(b * T + t) * d + k];
        __syncthreads();
        red[threadIdx.x] = acc;
        __syncthreads();
        if (r == 0 && k < d) partial[(size_t)(b * kSlices + slice) * d + k] = ((red[kk] + red[64 + kk]) + red[128 + kk]) + red[192 + kk];
    }
}

__global__ void steplog_final_kernel(const double *partial, double *lambda, int d, double scale)
{
    const long long b = blockIdx.x;
    for (int k = threadIdx.x; k < d; k += blockDim.x) {
        double acc = 0.0;
        for (int sl = 0; sl < kSlices; ++sl) acc += partial[(size_t)(b * kSlices + sl) * d + k];
        lambda[b * d + k] = acc * scale;
    }
}

// Largest exponent from the final vector v = J_T ... J_1 u_0 (paper Section 4.2.2):
// LSE(2 Re v') / (2 dt T); one thread per batch item.
template <typename R> __global__ void lle_epilogue_kernel(const R *v, double *lle, long long batch, int d, double scale)
{
    const long long b = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    const R *p = v + (size_t)b * d * 2;
    double m = -__builtin_huge_val();
    for (int i = 0; i < d; ++i) m = fmax(m, 2.0 * (double)p[2 * i]);
    if (!(m > -__builtin_huge_val())) {
        lle[b] = -__builtin_huge_val();
        return;
    }
    double acc = 0.0;
    for (int i = 0; i < d; ++i) acc += exp(2.0 * (double)p[2 * i] - m);
    lle[b] = (m + log(acc)) * scale;
}

// u_0 = (1, ..., 1) / sqrt(d) as GOOMs
template <typename R> __global__ void uniform_u0_kernel(R *u, long long n, int d)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    u[2 * i] = (R)(-0.5 * log((double)d));
    u[2 * i + 1] = (R)0;
}

// After phase 3 has stored the states of every chunk: the state at a reset step is the
// reset one, which is the prefix entering the next chunk; also fills the per-step flags.
struct ResetPostArgs {
    const unsigned char *carries; // factored prefixes with double mantissas
    long long car_stride;
    int car_cols;
    int dp;
    const unsigned char *chunk_flags;
    void *states;         // NULL or [batch][T][d][d] GOOMs
    unsigned char *flags; // NULL or [batch][T]
    long long T, L, C;
    int d;
};

template <typename IO> __global__ __launch_bounds__(kThreads) void reset_post_kernel(ResetPostArgs a)
{
    const long long b = blockIdx.x / a.C, c = blockIdx.x % a.C;
    const int tid = threadIdx.x, d = a.d;
    const long long t_first = c * a.L;
    long long len = a.T - t_first;
    if (len > a.L) len = a.L;
    const bool was_reset = a.chunk_flags[b * a.C + c] != 0;
    if (a.flags)
        for (long long t = tid; t < len; t += kThreads) a.flags[b * a.T + t_first + t] = (was_reset && t == len - 1) ? 1 : 0;
    if (!was_reset || !a.states) return;
    const unsigned char *src = a.carries + (b * (a.C + 1) + c + 1) * a.car_stride;
    const double *mp = reinterpret_cast<const double *>(src);
    const double *ep = reinterpret_cast<const double *>(src + (size_t)a.dp * a.car_cols * sizeof(double));
    IO *op = static_cast<IO *>(a.states) + ((size_t)(b * a.T + t_first + len - 1) * d * d) * 2;
    const IO pi = sizeof(IO) == 4 ? (IO)3.14159274101257324219f : (IO)3.14159265358979311600;
    for (int e = tid; e < d * d; e += kThreads) {
        const int i = e / d, k = e % d;
        const double v = mp[(size_t)i * a.car_cols + k];
        const double re = v != 0.0 ? log(fabs(v)) + ep[k] * kLn2 : -__builtin_huge_val();
        op[(size_t)e * 2] = (IO)re;
        op[(size_t)e * 2 + 1] = v < 0.0 ? pi : (IO)0;
    }
}

} // namespace

namespace goom {

int launch_reset_post(goom_ctx *ctx, const ResetLaunch &l)
{
    ResetPostArgs a;
    a.carries = static_cast<const unsigned char *>(l.carries);
    a.car_stride = l.car_stride;
    a.car_cols = l.car_cols;
    a.dp = padded_dim(l.d);
    a.chunk_flags = l.chunk_flags;
    a.states = l.post_states;
    a.flags = l.flags;
    a.T = l.T;
    a.L = l.L;
    a.C = l.C;
    a.d = l.d;
    const long long grid = l.batch * l.C;
    if (grid > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "too many chunks for one launch");
    prof_begin(ctx, "reset_post_states_flags");
    if (l.dtype == GOOM_C64)
        hipLaunchKernelGGL(reset_post_kernel<float>, dim3((unsigned)grid), dim3(kThreads), 0, ctx->stream, a);
    else
        hipLaunchKernelGGL(reset_post_kernel<double>, dim3((unsigned)grid), dim3(kThreads), 0, ctx->stream, a);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch reset_post_kernel");
}


int launch_lyap_steps(goom_ctx *ctx, const void *J, const void *S0, const void *states, double *steplog, double *partial,
                      double *lambda, long long T, int d, long long batch, int dtype, double scale)
{
    const long long grid = batch * T;
    if (grid > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "too many steps for one launch");
    const int dp = padded_dim(d);
    if (d > 128) return fail(ctx, GOOM_EUNSUPPORTED, "the per-step estimator supports d <= 128 (d=%d)", d);
    prof_begin(ctx, "lyapunov_per_step_qr");
    if (dp == 128) { // four waves per step
        const size_t lds = (size_t)8 * 128 * 18 * sizeof(double) + sizeof(WideScratch);
        const void *kern = dtype == GOOM_C64 ? reinterpret_cast<const void *>(lyap_step_wide_kernel<float>) : reinterpret_cast<const void *>(lyap_step_wide_kernel<double>);
        if (int st = check_hip(ctx, hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds), "hipFuncSetAttribute(lyap_step_wide_kernel)")) return st;
        if (dtype == GOOM_C64)
            hipLaunchKernelGGL(lyap_step_wide_kernel<float>, dim3((unsigned)grid), dim3(256), lds, ctx->stream, static_cast<const float *>(J),
                               static_cast<const float *>(S0), static_cast<const float *>(states), steplog, T, d);
        else
            hipLaunchKernelGGL(lyap_step_wide_kernel<double>, dim3((unsigned)grid), dim3(256), lds, ctx->stream, static_cast<const double *>(J),
                               static_cast<const double *>(S0), static_cast<const double *>(states), steplog, T, d);
    } else
    if (dtype == GOOM_C64) {
        StepArgs a;
        a.J = static_cast<const float *>(J);
        a.S0 = static_cast<const float *>(S0);
        a.states = static_cast<const float *>(states);
        a.steplog = steplog;
        a.T = T;
        a.d = d;
        if (dp == 16)
            hipLaunchKernelGGL(lyap_step_kernel<16>, dim3((unsigned)grid), dim3(64), 0, ctx->stream, a);
        else if (dp == 32)
            hipLaunchKernelGGL(lyap_step_kernel<32>, dim3((unsigned)grid), dim3(64), 0, ctx->stream, a);
        else
            hipLaunchKernelGGL(lyap_step_kernel<64>, dim3((unsigned)grid), dim3(64), 0, ctx->stream, a);
    } else {
        StepArgsD a;
        a.J = static_cast<const double *>(J);
        a.S0 = static_cast<const double *>(S0);
        a.states = static_cast<const double *>(states);
        a.steplog = steplog;
        a.T = T;
        a.d = d;
        if (dp == 16)
            hipLaunchKernelGGL(lyap_step_kernel_d<16>, dim3((unsigned)grid), dim3(64), 0, ctx->stream, a);
        else if (dp == 32)
            hipLaunchKernelGGL(lyap_step_kernel_d<32>, dim3((unsigned)grid), dim3(64), 0, ctx->stream, a);
        else
            hipLaunchKernelGGL(lyap_step_kernel_d<64>, dim3((unsigned)grid), dim3(64), 0, ctx->stream, a);
    }
    prof_end(ctx);
    if (int st = check_hip(ctx, hipGetLastError(), "launch lyap_step_kernel")) return st;
    prof_begin(ctx, "lyapunov_mean_of_logs");
    hipLaunchKernelGGL(steplog_partial_kernel, dim3((unsigned)(batch * kSlices)), dim3(256), 0, ctx->stream, steplog, partial, T, d);
    hipLaunchKernelGGL(steplog_final_kernel, dim3((unsigned)batch), dim3(64), 0, ctx->stream, partial, lambda, d, scale);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch steplog kernels");
}

size_t lyap_steps_partial_bytes(long long batch, int d) { return align_up((size_t)batch * kSlices * d * sizeof(double), 256); }

int launch_lle_epilogue(goom_ctx *ctx, const void *v, double *lle, long long batch, int d, int dtype, double scale)
{
    const unsigned blocks = (unsigned)((batch + 63) / 64);
    prof_begin(ctx, "lle_log_norm");
    if (dtype == GOOM_C64)
        hipLaunchKernelGGL(lle_epilogue_kernel<float>, dim3(blocks), dim3(64), 0, ctx->stream, static_cast<const float *>(v), lle, batch, d, scale);
    else
        hipLaunchKernelGGL(lle_epilogue_kernel<double>, dim3(blocks), dim3(64), 0, ctx->stream, static_cast<const double *>(v), lle, batch, d, scale);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch lle_epilogue_kernel");
}

int launch_uniform_u0(goom_ctx *ctx, void *u, long long batch, int d, int dtype)
{
    const long long n = batch * d;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    if (dtype == GOOM_C64)
        hipLaunchKernelGGL(uniform_u0_kernel<float>, dim3(blocks), dim3(256), 0, ctx->stream, static_cast<float *>(u), n, d);
    else
        hipLaunchKernelGGL(uniform_u0_kernel<double>, dim3(blocks), dim3(256), 0, ctx->stream, static_cast<double *>(u), n, d);
    return check_hip(ctx, hipGetLastError(), "launch uniform_u0_kernel");
}

size_t reset_tree_workspace_bytes(long long T, int d, long long batch, int dtype)
{
    const size_t mat = (size_t)d * d * 2 * (dtype == GOOM_C64 ? 4 : 8);
    return align_up((size_t)batch * (T + 1) * mat, 256) + align_up((size_t)(T + 1) * mat, 256) + align_up((size_t)batch * (T + 1), 256);
}

template <typename IO> static int run_reset_tree_t(goom_ctx *ctx, const void *J, const void *S0, void *states, unsigned char *out_flags, long long T, int d,
                                                   long long batch, int dtype, int policy, float cos_threshold, void *ws)
{
    const long long n = T + 1;
    const size_t mat = (size_t)d * d * 2 * sizeof(IO);
    unsigned char *w = static_cast<unsigned char *>(ws);
    unsigned char *Mall = w;
    unsigned char *tmp = w + align_up((size_t)batch * n * mat, 256);
    unsigned char *flags = tmp + align_up((size_t)n * mat, 256);
    const int dp = padded_dim(d);
    if (n > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "too many steps for one launch");
    const size_t wide_lds = (size_t)8 * 128 * 18 * sizeof(double) + sizeof(WideScratch);
    if (dp == 128)
        if (int st = check_hip(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(tree_reset_wide_kernel<IO>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)wide_lds),
                               "hipFuncSetAttribute(tree_reset_wide_kernel)"))
            return st;
    for (long long b = 0; b < batch; ++b) {
        IO *M = reinterpret_cast<IO *>(Mall + (size_t)b * n * mat);
        unsigned char *flag = flags + (size_t)b * n;
        hipLaunchKernelGGL(tree_init_kernel<IO>, dim3((unsigned)n), dim3(256), 0, ctx->stream, static_cast<const IO *>(J) + (size_t)b * T * d * d * 2,
                           S0 ? static_cast<const IO *>(S0) + (size_t)b * d * d * 2 : nullptr, M, flag, n, d);
        for (long long half = 1; half < n; half *= 2) {
            TreeResetArgs a;
            a.M = M;
            a.flag = flag;
            a.n = n;
            a.d = d;
            a.policy = policy;
            a.cos_threshold = cos_threshold;
            prof_begin(ctx, "reset_tree_select_and_reset");
            if (dp == 16) hipLaunchKernelGGL((tree_reset_kernel<16, IO>), dim3((unsigned)n), dim3(64), 0, ctx->stream, a);
            else if (dp == 32) hipLaunchKernelGGL((tree_reset_kernel<32, IO>), dim3((unsigned)n), dim3(64), 0, ctx->stream, a);
            else if (dp == 64) hipLaunchKernelGGL((tree_reset_kernel<64, IO>), dim3((unsigned)n), dim3(64), 0, ctx->stream, a);
            else hipLaunchKernelGGL(tree_reset_wide_kernel<IO>, dim3((unsigned)n), dim3(256), wide_lds, ctx->stream, a);
            prof_end(ctx);
            if (int st = check_hip(ctx, hipGetLastError(), "launch tree_reset_kernel")) return st;
            // products of this parallel step: whole blocks, then the ragged last one
            const long long full = n / (2 * half), rest = n % (2 * half) > half ? n % (2 * half) - half : 0;
            for (int part = 0; part < 2; ++part) {
                const long long items = part == 0 ? full : (rest ? 1 : 0), steps = part == 0 ? half : rest;
                if (items == 0) continue;
                const long long first = part == 0 ? 0 : full * 2 * half; // first element of the first block of this part
                ChainLaunch l;
                std::memset(&l, 0, sizeof l);
                l.dtype = dtype;
                l.n = l.d = l.m = d;
                l.left = reinterpret_cast<unsigned char *>(M) + (size_t)(first + half) * mat;
                l.left_batch_stride = (long long)(2 * half * mat);
                l.left_step_stride = (long long)mat;
                l.steps = steps;
                l.chunk_len = 1;
                l.chunks_launched = steps;
                l.batch = items;
                l.init_mode = 2;
                l.init = reinterpret_cast<unsigned char *>(M) + (size_t)(first + half - 1) * mat;
                l.init_stride = (long long)(2 * half * mat);
                l.out_goom = tmp + (size_t)(part == 0 ? 0 : full * half) * mat;
                l.label = "reset_tree_products";
                if (int st = launch_chain(ctx, l)) return st;
            }
            const long long updated = full * half + rest;
            if (updated > 0)
                hipLaunchKernelGGL(tree_scatter_kernel<IO>, dim3((unsigned)updated), dim3(256), 0, ctx->stream, M, reinterpret_cast<const IO *>(tmp), flag, n, d, half);
            if (int st = check_hip(ctx, hipGetLastError(), "launch tree_scatter_kernel")) return st;
        }
        hipLaunchKernelGGL(tree_finish_kernel<IO>, dim3((unsigned)T), dim3(256), 0, ctx->stream, M, flag, static_cast<IO *>(states) + (size_t)b * T * d * d * 2,
                           out_flags ? out_flags + (size_t)b * T : nullptr, n, d);
        if (int st = check_hip(ctx, hipGetLastError(), "launch tree_finish_kernel")) return st;
    }
    return GOOM_OK;
}

int run_reset_tree(goom_ctx *ctx, const void *J, const void *S0, void *states, unsigned char *out_flags, long long T, int d, long long batch,
                   int dtype, int policy, float cos_threshold, void *ws)
{
    return dtype == GOOM_C64 ? run_reset_tree_t<float>(ctx, J, S0, states, out_flags, T, d, batch, dtype, policy, cos_threshold, ws)
                             : run_reset_tree_t<double>(ctx, J, S0, states, out_flags, T, d, batch, dtype, policy, cos_threshold, ws);
}

int launch_reset_carry(goom_ctx *ctx, const ResetLaunch &l)
{
    ResetArgs a;
    a.totals = static_cast<const unsigned char *>(l.totals);
    a.tot_stride = l.tot_stride;
    a.tot_cols = l.tot_cols;
    a.carries = static_cast<unsigned char *>(l.carries);
    a.car_stride = l.car_stride;
    a.car_cols = l.car_cols;
    a.s0 = l.s0;
    a.chunk_flags = l.chunk_flags;
    a.growth = l.growth;
    a.growth_scale = l.growth_scale;
    a.T = l.T;
    a.L = l.L;
    a.C = l.C;
    a.d = l.d;
    a.policy = l.policy;
    a.cos_threshold = l.cos_threshold;
    const int dp = padded_dim(l.d);
    if (l.d > 128) return fail(ctx, GOOM_EUNSUPPORTED, "the reset scan supports d <= 128 (d=%d)", l.d);
    if (dp == 128) { // four waves per batch item, the state's columns divided among them
        const size_t lds = (size_t)8 * 128 * 18 * sizeof(double) + sizeof(WideScratch);
        const void *kern = l.dtype == GOOM_C64 ? reinterpret_cast<const void *>(reset_carry_wide_kernel<float>) : reinterpret_cast<const void *>(reset_carry_wide_kernel<double>);
        if (int st = check_hip(ctx, hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds), "hipFuncSetAttribute(reset_carry_wide_kernel)")) return st;
        prof_begin(ctx, "reset_phase2_carries_qr");
        if (l.dtype == GOOM_C64)
            hipLaunchKernelGGL(reset_carry_wide_kernel<float>, dim3((unsigned)l.batch), dim3(256), lds, ctx->stream, a);
        else
            hipLaunchKernelGGL(reset_carry_wide_kernel<double>, dim3((unsigned)l.batch), dim3(256), lds, ctx->stream, a);
        prof_end(ctx);
        return check_hip(ctx, hipGetLastError(), "launch reset_carry_wide_kernel");
    }
    prof_begin(ctx, "reset_phase2_carries_qr");
#define GOOM_RESET_CASE(DPV)                                                                                                   \
    if (dp == DPV) {                                                                                                           \
        if (l.dtype == GOOM_C64)                                                                                               \
            hipLaunchKernelGGL((reset_carry_kernel<DPV, float>), dim3((unsigned)l.batch), dim3(64), 0, ctx->stream, a);       \
        else                                                                                                                   \
            hipLaunchKernelGGL((reset_carry_kernel<DPV, double>), dim3((unsigned)l.batch), dim3(64), 0, ctx->stream, a);      \
    }
    GOOM_RESET_CASE(16)
    GOOM_RESET_CASE(32)
    GOOM_RESET_CASE(64)
#undef GOOM_RESET_CASE
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch reset_carry_kernel");
}

} // namespace goom
