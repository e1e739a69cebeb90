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
// final state, so growth / (dt T) is the Lyapunov spectrum (paper eq. 12, with the
// triangular factors taken at the resets: triangular factors multiply, so their diagonals
// accumulate exactly as in the step-by-step method).
//
// One workgroup of 256 threads; everything lives in LDS; float arithmetic with double
// accumulation of the logarithms.  The chain of chunks is inherently serial (each reset
// depends on the previous one), so this phase is latency bound; it is small next to the
// streaming phases as long as the chunk count stays in the hundreds.
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
    const float *s0;             // NULL or GOOM initial state [batch][d][d]
    unsigned char *chunk_flags;  // [batch][C]: 1 where the state at the end of chunk c was reset
    double *growth;              // NULL or [batch][d]
    double growth_scale;         // 1, or 1 / (dt T) to return exponents
    long long T, L, C;
    int d;
    int policy;
    float cos_threshold;
};

__device__ inline float warp_sum(float v)
{
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
    return v;
}

// Column-major d x d matrix in LDS with leading dimension LD = DP + 1.
template <int DP> struct Lds {
    static constexpr int LD = DP + 1;
    float t[DP * LD];   // chunk product (row-major here: t[i * LD + j])
    float y[DP * LD];   // state, column-major: y[k * LD + i]
    float z[DP * LD];   // product / work, column-major
    float rdiag[DP];    // diagonal of R
    float colscale[DP]; // per-column scalars
    double yexp[DP];    // power-of-two exponent of every state column
    double lognorm[DP]; // natural log of every column norm of z (including exponents)
    int flag;
};

// Right-looking modified Gram-Schmidt on the columns of m (column-major, d x d), in place:
// m <- Q, rdiag <- diag(R) (> 0).  Returns nothing; a zero column stays zero with R_kk = 0.
template <int DP> __device__ void mgs_sweep(float *m, float *rdiag, float *tmp, int d, int tid)
{
    constexpr int LD = DP + 1;
    const int lane = tid & 63, wave = tid >> 6;
    for (int k = 0; k < d; ++k) {
        // norm of column k (first wave)
        if (wave == 0) {
            float v = lane < d ? m[k * LD + lane] : 0.0f;
            float ss = warp_sum(v * v);
            float nrm = __builtin_sqrtf(ss);
            if (lane == 0) rdiag[k] = nrm;
            if (lane < d) m[k * LD + lane] = nrm > 0.0f ? v / nrm : 0.0f;
        }
        __syncthreads();
        // r_kj = q_k . a_j for j > k: 8 threads per column j, then a_j -= r_kj q_k
        const int nrem = d - 1 - k;
        for (int j0 = 0; j0 < nrem; j0 += kThreads / 8) {
            const int jj = j0 + (tid >> 3);
            const int j = k + 1 + jj;
            const int part = tid & 7;
            float dot = 0.0f;
            if (jj < nrem)
                for (int i = part; i < d; i += 8) dot += m[k * LD + i] * m[j * LD + i];
            dot += __shfl_xor(dot, 1, 64);
            dot += __shfl_xor(dot, 2, 64);
            dot += __shfl_xor(dot, 4, 64);
            if (jj < nrem && part == 0) tmp[j] = dot;
        }
        __syncthreads();
        for (int e = tid; e < nrem * d; e += kThreads) {
            const int j = k + 1 + e / d, i = e % d;
            m[j * LD + i] -= tmp[j] * m[k * LD + i];
        }
        __syncthreads();
    }
}

template <int DP> __global__ __launch_bounds__(kThreads) void reset_carry_kernel(ResetArgs a)
{
    constexpr int LD = DP + 1;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    Lds<DP> &s = *reinterpret_cast<Lds<DP> *>(smem_raw);
    const int tid = threadIdx.x;
    const int d = a.d;
    const long long b = blockIdx.x;
    const size_t tot_mant = (size_t)DP * a.tot_cols * sizeof(float);
    const size_t car_mant = (size_t)DP * a.car_cols * sizeof(float);
    double growth_acc = 0.0; // thread k < d accumulates column k

    // ---- initial state Y_0: identity or the given GOOM matrix, columns scaled by powers of two
    for (int e = tid; e < DP * LD; e += kThreads) s.y[e] = 0.0f;
    if (tid < DP) s.yexp[tid] = 0.0;
    __syncthreads();
    if (!a.s0) {
        if (tid < d) s.y[tid * LD + tid] = 1.0f;
    } else {
        const float *gp = a.s0 + (size_t)b * d * d * 2;
        if (tid < d) { // column tid
            float cmax = -__builtin_huge_valf();
            for (int i = 0; i < d; ++i) cmax = fmaxf(cmax, gp[((size_t)i * d + tid) * 2]);
            s.yexp[tid] = cmax > -__builtin_huge_valf() ? ceil((double)cmax * kLog2e) : 0.0;
        }
        __syncthreads();
        for (int e = tid; e < d * d; e += kThreads) {
            const int i = e / d, k = e % d;
            const double t = (double)gp[(size_t)e * 2] * kLog2e - s.yexp[k];
            float v = t > -300.0 ? (float)exp2(t) : 0.0f;
            const int par = (int)rintf(gp[(size_t)e * 2 + 1] * 0.318309886183790671538f);
            s.y[k * LD + i] = (par & 1) ? -v : v;
        }
    }
    __syncthreads();

    auto store_carry = [&](long long c) {
        unsigned char *dst = a.carries + (b * (a.C + 1) + c) * a.car_stride;
        float *mp = reinterpret_cast<float *>(dst);
        double *ep = reinterpret_cast<double *>(dst + car_mant);
        for (int e = tid; e < DP * a.car_cols; e += kThreads) {
            const int i = e / a.car_cols, k = e % a.car_cols;
            mp[e] = (i < d && k < d) ? s.y[k * LD + i] : 0.0f;
        }
        if (tid < a.car_cols) ep[tid] = tid < d ? s.yexp[tid] : 0.0;
    };

    // normalise the columns of z to unit norm: z <- z / |z_k|, lognorm_k = ln|z_k| + ln 2 * (exponent of column k)
    auto normalise_z = [&](const double *col_exp) {
        const int lane = tid & 63, wave = tid >> 6;
        for (int k = wave; k < d; k += kThreads / 64) {
            float v = lane < d ? s.z[k * LD + lane] : 0.0f;
            // scale by the largest entry first so that the squares cannot under/overflow
            float mx = fabsf(v);
#pragma unroll
            for (int sft = 32; sft >= 1; sft >>= 1) mx = fmaxf(mx, __shfl_xor(mx, sft, 64));
            int ex = 0;
            if (mx > 0.0f) (void)frexpf(mx, &ex);
            v = ldexpf(v, -ex);
            const float ss = warp_sum(v * v);
            const float nrm = __builtin_sqrtf(ss);
            if (lane < d) s.z[k * LD + lane] = nrm > 0.0f ? v / nrm : 0.0f;
            if (lane == 0)
                s.lognorm[k] = nrm > 0.0f ? log((double)nrm) + ((double)ex + col_exp[k]) * kLn2 : -__builtin_huge_val();
        }
        __syncthreads();
    };

    // does any pair of unit columns of z have |cosine| above the threshold?
    auto near_colinear = [&]() {
        if (tid == 0) s.flag = 0;
        __syncthreads();
        int hit = 0;
        for (int e = tid; e < d * d; e += kThreads) {
            const int p = e / d, q = e % d;
            if (p < q) {
                float dot = 0.0f;
                for (int i = 0; i < d; ++i) dot += s.z[p * LD + i] * s.z[q * LD + i];
                if (fabsf(dot) > a.cos_threshold) hit = 1;
            }
        }
        if (hit) s.flag = 1;
        __syncthreads();
        return s.flag != 0;
    };

    // QR of z (unit columns) by two Gram-Schmidt sweeps; z <- Q, colscale <- diag(R)
    auto qr_z = [&]() {
        mgs_sweep<DP>(s.z, s.rdiag, s.colscale, d, tid);
        if (tid < d) s.t[tid] = s.rdiag[tid]; // first sweep's diagonal (t is free here)
        __syncthreads();
        mgs_sweep<DP>(s.z, s.rdiag, s.colscale, d, tid); // second sweep restores orthogonality; its R is near identity
        if (tid < d) s.colscale[tid] = s.t[tid] * s.rdiag[tid];
        __syncthreads();
    };

    for (long long c = 0; c < a.C; ++c) {
        store_carry(c);
        // ---- Z = T_c Y
        const unsigned char *tp = a.totals + (b * a.C + c) * a.tot_stride;
        const float *tm = reinterpret_cast<const float *>(tp);
        const double tex = *reinterpret_cast<const double *>(tp + tot_mant);
        for (int e = tid; e < d * d; e += kThreads) {
            const int i = e / d, j = e % d;
            s.t[i * LD + j] = tm[(size_t)i * a.tot_cols + j];
        }
        __syncthreads();
        for (int e = tid; e < d * d; e += kThreads) {
            const int k = e / d, i = e % d; // consecutive threads walk down a column
            float acc = 0.0f;
            for (int j = 0; j < d; ++j) acc += s.t[i * LD + j] * s.y[k * LD + j];
            s.z[k * LD + i] = acc;
        }
        __syncthreads();
        const long long t_end = (c + 1) * a.L; // 1-based step this chunk ends at (if it is a full chunk)
        const bool boundary = t_end <= a.T && a.policy >= 0;
        bool did_reset = false;
        if (boundary) {
            // exponents of z's columns: chunk product's common exponent + the state's
            if (tid < d) s.colscale[tid] = 0.0f;
            __syncthreads();
            // keep an unnormalised copy in y for the no-reset case: y <- z happens below
            // normalise a copy: we normalise z in place and remember the scale to undo it if needed
            // (col_exp = tex + yexp)
            if (tid < d) s.yexp[tid] += tex;
            __syncthreads();
            // save z before normalising (into t, which is free now) in case no reset happens
            for (int e = tid; e < DP * LD; e += kThreads) s.t[e] = s.z[e];
            __syncthreads();
            normalise_z(s.yexp);
            did_reset = a.policy == 1 || near_colinear();
            if (did_reset) {
                qr_z();
                if (tid < d && s.colscale[tid] > 0.0f) growth_acc += log((double)s.colscale[tid]) + s.lognorm[tid];
                for (int e = tid; e < DP * LD; e += kThreads) s.y[e] = s.z[e];
                if (tid < d) s.yexp[tid] = 0.0;
                __syncthreads();
            } else {
                for (int e = tid; e < DP * LD; e += kThreads) s.z[e] = s.t[e]; // restore the product
                __syncthreads();
            }
        } else {
            if (tid < d) s.yexp[tid] += tex;
            __syncthreads();
        }
        if (tid == 0) a.chunk_flags[b * a.C + c] = did_reset ? 1 : 0;
        if (!did_reset) {
            // Y <- Z with every column renormalised by a power of two
            const int lane = tid & 63, wave = tid >> 6;
            for (int k = wave; k < d; k += kThreads / 64) {
                float v = lane < d ? s.z[k * LD + lane] : 0.0f;
                float mx = fabsf(v);
#pragma unroll
                for (int sft = 32; sft >= 1; sft >>= 1) mx = fmaxf(mx, __shfl_xor(mx, sft, 64));
                int ex = 0;
                if (mx > 0.0f) (void)frexpf(mx, &ex);
                if (lane < d) s.y[k * LD + lane] = ldexpf(v, -ex);
                if (lane == 0) s.yexp[k] += (double)ex;
            }
            __syncthreads();
        }
    }

    store_carry(a.C); // the final state
    __syncthreads();

    // ---- growth of the final state (factorised, not replaced)
    if (a.growth) {
        for (int e = tid; e < DP * LD; e += kThreads) s.z[e] = s.y[e];
        __syncthreads();
        normalise_z(s.yexp);
        qr_z();
        if (tid < d) {
            if (s.colscale[tid] > 0.0f) growth_acc += log((double)s.colscale[tid]) + s.lognorm[tid];
            a.growth[b * d + tid] = growth_acc * a.growth_scale;
        }
    }
}

// After phase 3 has stored the states of every chunk: the state at a reset step is the
// reset one, which is the prefix entering the next chunk; also fills the per-step flags.
struct ResetPostArgs {
    const unsigned char *carries;
    long long car_stride;
    int car_cols;
    int dp;
    const unsigned char *chunk_flags;
    float *states;        // NULL or [batch][T][d][d] GOOMs
    unsigned char *flags; // NULL or [batch][T]
    long long T, L, C;
    int d;
};

__global__ __launch_bounds__(kThreads) void reset_post_kernel(ResetPostArgs a)
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
    const float *mp = reinterpret_cast<const float *>(src);
    const double *ep = reinterpret_cast<const double *>(src + (size_t)a.dp * a.car_cols * sizeof(float));
    float *op = a.states + ((size_t)(b * a.T + t_first + len - 1) * d * d) * 2;
    for (int e = tid; e < d * d; e += kThreads) {
        const int i = e / d, k = e % d;
        const float v = mp[(size_t)i * a.car_cols + k];
        const double re = v != 0.0f ? (log2((double)fabsf(v)) + ep[k]) * kLn2 : -__builtin_huge_val();
        op[(size_t)e * 2] = (float)re;
        op[(size_t)e * 2 + 1] = v < 0.0f ? 3.14159274101257324219f : 0.0f;
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
    a.states = static_cast<float *>(l.post_states);
    a.flags = l.flags;
    a.T = l.T;
    a.L = l.L;
    a.C = l.C;
    a.d = l.d;
    const long long grid = l.batch * l.C;
    if (grid > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "too many chunks for one launch");
    prof_begin(ctx, "reset_post_states_flags");
    hipLaunchKernelGGL(reset_post_kernel, dim3((unsigned)grid), dim3(kThreads), 0, ctx->stream, a);
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch reset_post_kernel");
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
    a.s0 = static_cast<const float *>(l.s0);
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
    prof_begin(ctx, "reset_phase2_carries_qr");
    if (dp == 16) {
        hipLaunchKernelGGL(reset_carry_kernel<16>, dim3((unsigned)l.batch), dim3(kThreads), sizeof(Lds<16>), ctx->stream, a);
    } else if (dp == 32) {
        hipLaunchKernelGGL(reset_carry_kernel<32>, dim3((unsigned)l.batch), dim3(kThreads), sizeof(Lds<32>), ctx->stream, a);
    } else if (dp == 64) {
        auto kern = reset_carry_kernel<64>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)sizeof(Lds<64>));
        if (e != hipSuccess) return check_hip(ctx, e, "hipFuncSetAttribute(reset_carry_kernel)");
        hipLaunchKernelGGL(kern, dim3((unsigned)l.batch), dim3(kThreads), sizeof(Lds<64>), ctx->stream, a);
    } else {
        return fail(ctx, GOOM_EUNSUPPORTED, "the reset scan supports d <= 64 (d=%d)", l.d);
    }
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch reset_carry_kernel");
}

} // namespace goom
