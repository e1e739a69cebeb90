// chain kernel instantiations: float components, left factors as GOOMs
#include "goom_chain_fast.h"

namespace goom_chain {
int dispatch_f32_goom(goom_ctx *ctx, const ChainArgs &args, int dp, int nw, long long grid, const char *label)
{
    if (args.acc_f64) return dispatch_affine_chunk_f64(ctx, args, dp, grid, label);
    if (args.fact_f64 && !affine_walk_applies(args, dp)) return goom::fail(ctx, GOOM_EUNSUPPORTED, "double carries are read by the matrix-vector walk only");
    if (small_applies(args, dp)) return dispatch_small(ctx, args, grid, label);
    if (fast_applies(args, dp, nw)) return dispatch_fast(ctx, args, dp, grid, label);
    if (ragged_applies(args, dp, nw)) return dispatch_ragged(ctx, args, dp, grid, label);
    if (args.left_real) return goom::fail(ctx, GOOM_EUNSUPPORTED, "real left factors are read by the hot float kernel only (d = 32, 64 or 128, square state)");
    if (affine_chunk_applies(args, dp)) return dispatch_affine_chunk(ctx, args, dp, grid, label);
    if (affine_walk_applies(args, dp)) return dispatch_affine_walk(ctx, args, dp, grid, label);
    if (args.out_scaled) return goom::fail(ctx, GOOM_EUNSUPPORTED, "scaled outputs are written by the matrix-vector walk only (d = 16 or 32)");
    return dispatch<float, 0>(ctx, args, dp, nw, grid, label);
}
} // namespace goom_chain
