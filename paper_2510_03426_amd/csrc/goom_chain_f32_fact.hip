// chain kernel instantiations: float components, left factors factored
#include "goom_chain_kernel.h"

namespace goom_chain {
int dispatch_f32_fact(goom_ctx *ctx, const ChainArgs &args, int dp, int nw, long long grid, const char *label)
{
    return dispatch<float, 1>(ctx, args, dp, nw, grid, label);
}
} // namespace goom_chain
