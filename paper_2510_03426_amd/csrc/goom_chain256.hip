// Chains of matrices with 128 < d <= 256 (paper Section 4.1 runs its chains up to 1024 x 1024;
// this is the largest size whose running product still fits one compute unit's registers).
//
// The state d x m of a chain is split into halves of 128 columns; one workgroup of eight waves (two
// per SIMD, which together use the whole register file: one workgroup per compute unit) owns a half,
// wave w the 16-column slab 16 w .. 16 w + 15 of it for all 256 (padded) rows, in the accumulator
// layout of the 16 x 16 x 4 matrix instruction, so that one step's result is the next step's B operand
// without moving.  The left factor A_t is exponentiated block by block (32 of its columns at a time,
// i.e. 32 values of the contraction index) into a double-buffered LDS tile by all 512 threads, the
// block after it waiting in registers; the row shifts n_i of A_t
// (the identity of Section 3.2, eq. 12, allows any: a whole number near the row's largest log2 magnitude) come from a pass of their own over
// the input, so a block can be converted before the rest of its rows has been seen.  After the
// eight blocks of a step the state is renormalised: row shifts folded into the mantissas, one
// power-of-two exponent per column (double).  A step costs 1024 matrix instructions per wave, which
// dominate everything else at this size.
//
// States enter and leave in the layout of the large-shape scan driver: transposed float mantissas
// St[state column][row] with one double exponent per state column.
#include "goom_internal.h"
#include "goom_chain_kernel.h"

namespace {

using goom_chain::Comp;
using goom_chain::f4;

constexpr int kDP = 256;          // padded matrix size
constexpr int kKB = 32;           // contraction indices per block
constexpr int kLDA = kKB + 4;     // padded row of the LDS tile
constexpr int kBlocks = kDP / kKB;
constexpr int kSlabs = 1;                       // 16-column slabs of the state per wave
constexpr int kThreads256 = 64 * (8 / kSlabs);  // eight slabs = 128 state columns per workgroup

struct Chain256Args {
    const float2 *M;     // [batch][T][d][d] GOOMs
    const float *nrow;   // [batch][T][256] row shifts
    long long T, L, chunks; // chain length, chunk length, chunks per batch item this launch covers
    long long nchains;      // batch * chunks
    int d, m, halves, mp;   // state is d x m, m <= mp = 128 * halves
    const float *init_s;    // NULL (identity) or [chain][mp][256] transposed mantissas
    const double *init_e;   //                    [chain][mp] column exponents
    float *out_s;           // NULL or the final state of every chain, same layout
    double *out_e;
    float2 *P;              // NULL or every prefix, [batch][T][d][m] GOOMs
};

// n[b][t][i] = ceil(max_j log2|A_ij|) (0 for a row of zeros and for padding rows).  One wave per row.
__global__ __launch_bounds__(256) void row_shift256_kernel(const float2 *__restrict__ M, float *__restrict__ nrow, int d, long long nmat)
{
    const int lane = threadIdx.x & 63;
    const long long mat = blockIdx.x / (kDP / 4);
    const int row = (int)(blockIdx.x % (kDP / 4)) * 4 + (threadIdx.x >> 6);
    if (mat >= nmat) return;
    float mx = -__builtin_huge_valf();
    if (row < d) {
        const float2 *arow = M + ((size_t)mat * d + row) * d;
        float x[4]; // d <= 256: four entries per lane, all loads in flight together
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = lane + 64 * r < d ? arow[lane + 64 * r].x : -__builtin_huge_valf();
        mx = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
    }
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) mx = fmaxf(mx, __shfl_xor(mx, s, 64));
    if (lane == 0) nrow[(size_t)mat * kDP + row] = mx > -__builtin_huge_valf() ? ceilf(mx * 1.44269504088896340736f) : 0.0f;
}

__global__ __launch_bounds__(kThreads256, kSlabs == 1 ? 2 : 1) void chain256_kernel(Chain256Args a)
{
    typedef Comp<float> C;
    extern __shared__ __align__(16) unsigned char smem[];
    float *tiles = reinterpret_cast<float *>(smem);                        // [2][256][36]
    float *nsh_all = tiles + 2 * kDP * kLDA;                               // [2][256]
    auto tile_of = [&](int b) { return tiles + (size_t)b * kDP * kLDA; };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    // Workgroups are dealt to the eight XCDs in turn (each has its own L2).  The two halves of a chain
    // read the same matrices at the same time, so they are numbered eight apart: same XCD, same L2.
    long long chain = blockIdx.x / a.halves;
    int half = (int)(blockIdx.x % a.halves);
    if (a.halves == 2) { // (the grid is padded to a multiple of 16 workgroups)
        chain = (long long)(blockIdx.x >> 4) * 8 + (blockIdx.x & 7);
        half = (blockIdx.x >> 3) & 1;
    }
    if (chain >= a.nchains) return; // whole workgroup, before any barrier
    const long long item = chain / a.chunks, chunk = chain % a.chunks;
    const long long t0 = chunk * a.L;
    long long len = a.T - t0;
    if (len > a.L) len = a.L;
    const int col0 = half * 128 + wave * 16 * kSlabs + c; // state columns of this lane: col0 (+ 16, ...)
    const int d = a.d;

    // conversion: eight lanes share a row of a block (four adjacent entries each)
    constexpr int NQ = 4 * kSlabs;      // passes of kThreads256 / 8 rows each
    constexpr int RPQ = kThreads256 / 8;
    const int crow = tid >> 3, c4 = 4 * (tid & 7);
    // (rows below 128 and the first four blocks of columns always lie inside the matrix, since d > 128;
    // elsewhere an address is clamped into the matrix and the value replaced by a zero entry)
    float2 pre[NQ][4];
    float npre[NQ];
    const int jlim = d - c4; // entry e of block kb exists iff 32 kb + e < jlim
    auto load_block = [&](long long t, int kb) {
        const float2 *mat = a.M + ((size_t)(item * a.T + t0 + t) * d) * d;
        const float *nr = a.nrow + (size_t)(item * a.T + t0 + t) * kDP;
        const bool inside = kKB * kb + kKB <= d; // wave-uniform
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int row = crow + RPQ * q;
            const bool row_ok = RPQ * q + RPQ <= 128 || row < d;
            const float2 *rp = mat + (size_t)(row_ok ? row : d - 1) * d + c4;
            npre[q] = nr[row];
            if (inside) {
#pragma unroll
                for (int e = 0; e < 4; ++e) pre[q][e] = rp[kKB * kb + e];
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int off = kKB * kb + e;
                    pre[q][e] = rp[off < jlim ? off : jlim - 1 > 0 ? jlim - 1 : 0];
                    if (!(off < jlim)) pre[q][e] = float2{-__builtin_huge_valf(), 0.0f};
                }
            }
            if (!row_ok) {
#pragma unroll
                for (int e = 0; e < 4; ++e) pre[q][e] = float2{-__builtin_huge_valf(), 0.0f};
            }
        }
    };
    // tile[i][j] = (+-) 2^(log2|A_ij| - n_i)
    auto convert_block = [&](int buf, bool first_block, int parity) {
        const float kHi = 1.44269502162933349609375f; // float nearest log2(e)
        const float kLo = 1.925963033500011e-8f;      // log2(e) - kHi
        float *tile = tile_of(buf);
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int row = crow + RPQ * q;
            f4 y;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float t = __builtin_fmaf(pre[q][e].x, kHi, -npre[q]);
                t = __builtin_fmaf(pre[q][e].x, kLo, t);
                const float v = __builtin_amdgcn_exp2f(t); // 2^-inf = 0 covers zero entries and the padding
                const float kf = __builtin_fmaf(pre[q][e].y, 0.318309886183790671538f, 12582912.0f);
                y[e] = __builtin_bit_cast(float, __builtin_bit_cast(int, v) | (__builtin_bit_cast(int, kf) << 31));
            }
            *reinterpret_cast<f4 *>(&tile[row * kLDA + c4]) = y;
            if (first_block && c4 == 0) nsh_all[parity * kDP + row] = npre[q];
        }
    };

    // ---- initial state: st[s][kt][v] = W[16 kt + 4 g + v][col0 + 16 s]
    float st[kSlabs][16][4];
    double ecol[kSlabs] = {};
#pragma unroll
    for (int s = 0; s < kSlabs; ++s) {
        const int col = col0 + 16 * s;
        if (a.init_s) {
            const float *sp = a.init_s + ((size_t)chain * a.mp + col) * kDP + 4 * g;
#pragma unroll
            for (int kt = 0; kt < 16; ++kt) {
                const f4 v4 = *reinterpret_cast<const f4 *>(sp + 16 * kt);
#pragma unroll
                for (int v = 0; v < 4; ++v) st[s][kt][v] = v4[v];
            }
            ecol[s] = a.init_e[(size_t)chain * a.mp + col];
        } else {
#pragma unroll
            for (int kt = 0; kt < 16; ++kt)
#pragma unroll
                for (int v = 0; v < 4; ++v) st[s][kt][v] = (16 * kt + 4 * g + v == col && col < d) ? 1.0f : 0.0f;
        }
    }

    if (len > 0) {
        load_block(0, 0);
        convert_block(0, true, 0);
        load_block(0, 1);
    }
    __syncthreads();

    for (long long t = 0; t < len; ++t) {
        const int parity = (int)(t & 1);
        f4 acc[kSlabs][16];
#pragma unroll
        for (int s = 0; s < kSlabs; ++s)
#pragma unroll
            for (int mt = 0; mt < 16; ++mt) acc[s][mt] = f4{0, 0, 0, 0};
#pragma unroll
        for (int kb = 0; kb < kBlocks; ++kb) {
            const float *tile = tile_of(kb & 1);
            // ---------------------------------------------------- product over this block's contraction indices
#pragma unroll
            for (int ktl = 0; ktl < kKB / 16; ++ktl) {
#pragma unroll
                for (int mh = 0; mh < 4; ++mh) {
                    f4 av[4];
#pragma unroll
                    for (int mi = 0; mi < 4; ++mi)
                        av[mi] = *reinterpret_cast<const f4 *>(&tile[(16 * (4 * mh + mi) + c) * kLDA + 16 * ktl + 4 * g]);
#pragma unroll
                    for (int v = 0; v < 4; ++v)
#pragma unroll
                        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                            for (int s = 0; s < kSlabs; ++s)
                                acc[s][4 * mh + mi] = C::mfma(av[mi][v], st[s][2 * kb + ktl][v], acc[s][4 * mh + mi]);
                }
            }
            // ---------------------------------------------------- next block into the other buffer, the one after it into registers
            const bool last_block = kb == kBlocks - 1;
            if (!last_block) {
                convert_block((kb + 1) & 1, false, parity);
                if (kb + 2 < kBlocks) load_block(t, kb + 2);
                else if (t + 1 < len) load_block(t + 1, 0);
            } else if (t + 1 < len) {
                convert_block(0, true, parity ^ 1);
                load_block(t + 1, 1);
            }
            if (!last_block) __syncthreads();
        }
        const float *nsh = nsh_all + parity * kDP;
#pragma unroll
        for (int s = 0; s < kSlabs; ++s) {
            const int col = col0 + 16 * s;
            // -------------------------------------------------------- outputs: entry (i, col) is acc 2^(n_i + ecol)
            if (a.P && col < a.m) {
                float2 *outp = a.P + ((size_t)(item * a.T + t0 + t) * d) * a.m + col;
                const float ecol_f = (float)ecol[s];
                // (the row limit is re-read every step: 64 loop-invariant lane masks, one per store, would
                // otherwise be kept in scalar registers for the whole loop)
                int rowlim = d - 4 * g;
                asm volatile("" : "+v"(rowlim));
                int mm = a.m; // likewise the 64 row offsets
                asm volatile("" : "+s"(mm));
                float2 *rowp = outp + (size_t)(4 * g) * mm;
#pragma unroll
                for (int mt = 0; mt < 16; ++mt) {
                    const f4 nv = *reinterpret_cast<const f4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float x = acc[s][mt][v];
                        if (16 * mt + v < rowlim) rowp[(16 * mt + v) * mm] = float2{C::out_re_f(x, nv[v] + ecol_f), x < 0.0f ? C::pi() : 0.0f};
                    }
                }
            }
            // -------------------------------------------------------- state: row shifts folded in, one exponent per column
            float cm = -1.0e30f;
#pragma unroll
            for (int mt = 0; mt < 16; ++mt) {
                const f4 nv = *reinterpret_cast<const f4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (acc[s][mt][v] != 0.0f) cm = C::max_(cm, C::exponent_of(acc[s][mt][v]) + nv[v]);
            }
            cm = C::xor16_32_max(cm);
            const bool all_zero = !(cm > -1.0e29f);
            const float sc = all_zero ? 0.0f : cm;
#pragma unroll
            for (int mt = 0; mt < 16; ++mt) {
                const f4 nv = *reinterpret_cast<const f4 *>(&nsh[16 * mt + 4 * g]);
#pragma unroll
                for (int v = 0; v < 4; ++v) st[s][mt][v] = __builtin_ldexpf(acc[s][mt][v], (int)C::clamp_shift(nv[v] - sc));
            }
            ecol[s] = all_zero ? 0.0 : ecol[s] + (double)sc;
        }
        __syncthreads();
    }

    if (a.out_s) {
#pragma unroll
        for (int s = 0; s < kSlabs; ++s) {
            const int col = col0 + 16 * s;
            float *sp = a.out_s + ((size_t)chain * a.mp + col) * kDP + 4 * g;
#pragma unroll
            for (int kt = 0; kt < 16; ++kt) *reinterpret_cast<f4 *>(sp + 16 * kt) = f4{st[s][kt][0], st[s][kt][1], st[s][kt][2], st[s][kt][3]};
            if (g == 0) a.out_e[(size_t)chain * a.mp + col] = ecol[s];
        }
    }
}

} // namespace

namespace goom {

size_t chain256_lds_bytes() { return (size_t)2 * kDP * kLDA * sizeof(float) + (size_t)2 * kDP * sizeof(float); }

int launch_row_shifts256(goom_ctx *ctx, const void *M, float *nrow, int d, long long nmat)
{
    const long long grid = nmat * (kDP / 4);
    if (grid <= 0) return GOOM_OK;
    if (grid > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "too many matrices for one launch (%lld)", nmat);
    hipLaunchKernelGGL(row_shift256_kernel, dim3((unsigned)grid), dim3(256), 0, ctx->stream, static_cast<const float2 *>(M), nrow, d, nmat);
    return check_hip(ctx, hipGetLastError(), "launch row_shift256_kernel");
}

int launch_chain256(goom_ctx *ctx, const void *M, const float *nrow, long long T, long long L, long long chunks, long long batch, int d, int m,
                    const float *init_s, const double *init_e, float *out_s, double *out_e, void *P)
{
    Chain256Args a;
    a.M = static_cast<const float2 *>(M);
    a.nrow = nrow;
    a.T = T;
    a.L = L;
    a.chunks = chunks;
    a.d = d;
    a.m = m;
    a.halves = (m + 127) / 128;
    a.mp = 128 * a.halves;
    a.init_s = init_s;
    a.init_e = init_e;
    a.out_s = out_s;
    a.out_e = out_e;
    a.P = static_cast<float2 *>(P);
    a.nchains = batch * chunks;
    long long grid = a.nchains * a.halves;
    if (grid <= 0) return GOOM_OK;
    if (a.halves == 2) grid = (grid + 15) / 16 * 16;
    if (grid > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "too many chains for one launch");
    const size_t lds = chain256_lds_bytes();
    if (int s = check_hip(ctx, hipFuncSetAttribute(reinterpret_cast<const void *>(chain256_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                          "hipFuncSetAttribute(chain256_kernel)"))
        return s;
    hipLaunchKernelGGL(chain256_kernel, dim3((unsigned)grid), dim3(kThreads256), lds, ctx->stream, a);
    return check_hip(ctx, hipGetLastError(), "launch chain256_kernel");
}

} // namespace goom
