// Hot chain kernel for square matrices whose size d is a multiple of four strictly between the sizes it is
// built for (16 < d < 128, d not 32 or 64): the tile is padded to the next of 32, 64, 128 with zero rows and
// columns, and only the ceil(d / 16) blocks of sixteen rows and columns that hold entries are multiplied
// (paper Section 4.1 runs chains of d x d matrices; its sizes are powers of two, which the unpadded
// instantiations serve).
#include "goom_chain_fast.h"

namespace goom_chain {

bool ragged_applies(const ChainArgs &args, int dp, int nw)
{
    const int d = args.d;
    return args.n == d && args.m == d && d % 4 == 0 && d > 16 && d < dp && (dp == 32 || dp == 64 || dp == 128) && nw == dp / 16 &&
           args.bias_mode == 0 && args.out_fact_steps == nullptr && !args.left_real && !args.out_scaled;
}

template <int DP, int NW, int KD> static int launch_ragged(goom_ctx *ctx, const ChainArgs &args, long long grid, const char *label)
{
    constexpr int LDA = DP + 4;
    const size_t lds = 2 * ((size_t)DP * LDA * sizeof(float) + (size_t)DP * sizeof(float)) + 128;
    void (*kern)(ChainArgs) = chain_kernel_fast_ragged<DP, NW, KD>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return goom::check_hip(ctx, e, "hipFuncSetAttribute(chain_kernel_fast_ragged)");
    }
    if (grid <= 0) return GOOM_OK;
    if (grid > 0x7fffffffLL) return goom::fail(ctx, GOOM_EUNSUPPORTED, "too many chains for one launch (%lld)", grid);
    goom::prof_begin(ctx, label);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NW * 64), lds, ctx->stream, args);
    goom::prof_end(ctx);
    return goom::check_hip(ctx, hipGetLastError(), "launch chain_kernel_fast_ragged");
}

int dispatch_ragged(goom_ctx *ctx, const ChainArgs &args, int dp, long long grid, const char *label)
{
    const int kd = (args.d + 15) / 16;
    if (dp == 32) return launch_ragged<32, 2, 2>(ctx, args, grid, label);
    if (dp == 64) return kd == 3 ? launch_ragged<64, 4, 3>(ctx, args, grid, label) : launch_ragged<64, 4, 4>(ctx, args, grid, label);
    switch (kd) {
    case 5: return launch_ragged<128, 8, 5>(ctx, args, grid, label);
    case 6: return launch_ragged<128, 8, 6>(ctx, args, grid, label);
    case 7: return launch_ragged<128, 8, 7>(ctx, args, grid, label);
    default: return launch_ragged<128, 8, 8>(ctx, args, grid, label);
    }
}

} // namespace goom_chain
