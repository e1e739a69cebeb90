// Host side of the chain kernel: picks the instantiation and fills the kernel arguments.
#include "goom_chain_kernel.h"

using goom_chain::ChainArgs;

namespace goom {

FactLayout fact_layout(int dp, int m, int dtype)
{
    FactLayout f;
    f.rows_padded = dp;
    f.cols_padded = (m + 15) / 16 * 16;
    size_t comp = dtype == GOOM_C64 ? 4 : 8;
    f.mant_bytes = (size_t)f.rows_padded * f.cols_padded * comp;
    f.stride = align_up(f.mant_bytes + (size_t)f.cols_padded * sizeof(double), 256);
    return f;
}

int padded_dim(int d) { return d <= 16 ? 16 : d <= 32 ? 32 : d <= 64 ? 64 : 128; }

// Waves per workgroup: one per 16-column slab of the state, rounded up to a width the
// kernel is instantiated for.
static int pick_waves(int dp, int nslabs)
{
    const int kt = dp / 16;
    if (nslabs <= 1) return 1;
    if (nslabs <= kt) return kt;
    if (nslabs == kt + 1) return kt + 1;
    return -1;
}

int chain_padded_dim(int n, int d, int m)
{
    int dp = padded_dim(n > d ? n : d);
    while (dp < 128 && pick_waves(dp, (m + 15) / 16) < 0) dp *= 2;
    return dp;
}

int launch_chain(goom_ctx *ctx, const ChainLaunch &l)
{
    const int dp = l.dp ? l.dp : chain_padded_dim(l.n, l.d, l.m);
    const int nslabs = (l.m + 15) / 16;
    const int nw = pick_waves(dp, nslabs);
    if (nw < 0) return fail(ctx, GOOM_EUNSUPPORTED, "state of %d columns with d = %d is not supported", l.m, l.d);
    ChainArgs a;
    a.left = static_cast<const unsigned char *>(l.left);
    a.left_batch_stride = l.left_batch_stride;
    a.left_step_stride = l.left_step_stride;
    a.steps = l.steps;
    a.chunk_len = l.chunk_len;
    a.chunks_per_item = (l.steps + l.chunk_len - 1) / l.chunk_len;
    a.chunks_launched = l.chunks_launched;
    a.n = l.n;
    a.d = l.d;
    a.m = l.m;
    a.nslabs = nslabs;
    a.init_mode = l.init_mode;
    a.init = static_cast<const unsigned char *>(l.init);
    a.init_stride = l.init_stride;
    a.init_group = l.init_group;
    a.init_ngroups = l.init_ngroups;
    a.out_goom = static_cast<unsigned char *>(l.out_goom);
    a.out_goom_last_only = l.out_goom_last_only;
    a.out_fact_steps = static_cast<unsigned char *>(l.out_fact_steps);
    a.out_fact_final = static_cast<unsigned char *>(l.out_fact_final);
    a.final_common_exponent = l.final_common_exponent;
    a.fact_stride = l.fact_stride;
    a.fact_cols = l.fact_cols;
    a.left_fact_cols = l.left_fact_cols;
    a.bias_mode = l.bias_mode;
    a.bias_col = l.bias_col;
    a.bias = static_cast<const unsigned char *>(l.bias);
    a.left_real = l.left_real;
    a.out_scaled = static_cast<float *>(l.out_scaled);
    a.out_logscale = static_cast<float *>(l.out_logscale);
    a.fact_f64 = l.fact_f64;
    a.acc_f64 = l.acc_f64;
    a.left_shift = l.left_shift;
    a.io_shift = l.io_shift;
    if (l.io_shift && !(!l.left_fact && !l.left_real && !l.io_c64 && l.bias_mode == 1 && !l.left_shift && !l.out_scaled && !l.acc_f64))
        return fail(ctx, GOOM_EUNSUPPORTED, "rescaled bias and states: GOOM factors with GOOM bias vectors only");
    if (l.left_shift && !(l.dtype == GOOM_C64 && !l.left_fact && !l.left_real && !l.io_c64 && (l.acc_f64 || (l.m == 1 && l.fact_f64)) && l.left_step_stride >= 0))
        return fail(ctx, GOOM_EUNSUPPORTED, "transposed factors in reverse order: double chunk products and the walk beside them only");
    if ((l.fact_f64 || l.acc_f64) && (l.dtype != GOOM_C64 || l.left_fact))
        return fail(ctx, GOOM_EUNSUPPORTED, "double factored matrices beside float GOOMs: recurrence kernels only");
    if (a.out_scaled && (l.dtype != GOOM_C64 || l.left_fact))
        return fail(ctx, GOOM_EUNSUPPORTED, "scaled outputs are written by the float matrix-vector walk only");
    const long long grid = l.batch * l.chunks_launched;
    if (l.left_real && (l.dtype != GOOM_C64 || l.left_fact))
        return fail(ctx, GOOM_EUNSUPPORTED, "real left factors are read by the hot float kernel only");
    if (l.io_c64) {
        if (l.dtype != GOOM_C128 || l.left_fact || l.left_real || l.out_scaled)
            return fail(ctx, GOOM_EUNSUPPORTED, "complex64 data with a double running product: GOOM left factors only");
        return goom_chain::dispatch_f64_goom_io32(ctx, a, dp, nw, grid, l.label);
    }
    if (l.dtype == GOOM_C64)
        return l.left_fact ? goom_chain::dispatch_f32_fact(ctx, a, dp, nw, grid, l.label) : goom_chain::dispatch_f32_goom(ctx, a, dp, nw, grid, l.label);
    return l.left_fact ? goom_chain::dispatch_f64_fact(ctx, a, dp, nw, grid, l.label) : goom_chain::dispatch_f64_goom(ctx, a, dp, nw, grid, l.label);
}

} // namespace goom
