// chain kernel instantiations: double running product, left factors / initial state / bias / outputs as complex64 GOOMs
#include "goom_chain_kernel.h"

namespace goom_chain {
int dispatch_f64_goom_io32(goom_ctx *ctx, const ChainArgs &args, int dp, int nw, long long grid, const char *label)
{
    return dispatch<double, 0, float>(ctx, args, dp, nw, grid, label);
}
} // namespace goom_chain
