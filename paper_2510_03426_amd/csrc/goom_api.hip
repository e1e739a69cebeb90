// C ABI of libgoom (see include/goom.h): argument validation and the host-side drivers
// that turn one call into kernel launches.  No device memory is allocated here.
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>

#include "goom_internal.h"

// Scratch memory of goom_scan_static, the entry point for callers that cannot allocate: the scan's workspace
// (chunk products, carries, group products) lives here instead of in a caller-provided buffer.  Every device
// that loads the library holds its own copy at its own address; in host code the name is only a handle for
// hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[GOOM_STATIC_SCRATCH_BYTES];

namespace goom {

static thread_local std::string t_error;

// Address of `scratch` on `device`, resolved once per device with that device current.
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[64];
static bool g_scratch_done[64];
static std::string g_scratch_err[64];

static void resolve_scratch(goom_ctx *ctx)
{
    const int dev = ctx->device;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (dev < 64 && g_scratch_done[dev]) {
        ctx->scratch = g_scratch_ptr[dev];
        ctx->scratch_error = g_scratch_err[dev];
        return;
    }
    int prev = -1;
    void *ptr = nullptr;
    std::string err;
    hipError_t e = hipGetDevice(&prev);
    if (e == hipSuccess) e = hipSetDevice(dev);
    if (e == hipSuccess) e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) {
        ptr = nullptr;
        err = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e);
        (void)hipGetLastError();
    } else if (!aligned(ptr, 256)) {
        ptr = nullptr;
        err = "static scratch array is not 256-byte aligned";
    }
    if (prev >= 0) (void)hipSetDevice(prev);
    ctx->scratch = ptr;
    ctx->scratch_error = err;
    if (dev < 64) {
        g_scratch_ptr[dev] = ptr;
        g_scratch_err[dev] = err;
        g_scratch_done[dev] = true;
    }
}

const char *thread_error() { return t_error.c_str(); }

int fail(goom_ctx *ctx, int status, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    t_error = buf;
    if (ctx) ctx->last_error = buf;
    return status;
}

int check_hip(goom_ctx *ctx, hipError_t e, const char *what)
{
    if (e == hipSuccess) return GOOM_OK;
    return fail(ctx, GOOM_EHIP, "%s: %s", what, hipGetErrorString(e));
}

void prof_reset(goom_ctx *ctx)
{
    if (!ctx) return;
    for (auto &r : ctx->prof) ctx->prof_pool.push_back(r);
    ctx->prof.clear();
}

void prof_begin(goom_ctx *ctx, const char *label)
{
    if (!ctx || !ctx->profile) return;
    goom_prof_rec r;
    if (!ctx->prof_pool.empty()) {
        r = ctx->prof_pool.back();
        ctx->prof_pool.pop_back();
    } else {
        if (hipEventCreate(&r.start) != hipSuccess) return;
        if (hipEventCreate(&r.stop) != hipSuccess) { (void)hipEventDestroy(r.start); return; }
    }
    r.label = label ? label : "kernel";
    (void)hipEventRecord(r.start, ctx->stream);
    ctx->prof.push_back(r);
}

void prof_end(goom_ctx *ctx)
{
    if (!ctx || !ctx->profile || ctx->prof.empty()) return;
    (void)hipEventRecord(ctx->prof.back().stop, ctx->stream);
}

static size_t comp_bytes(int dtype) { return dtype == GOOM_C64 ? 4 : 8; }

static int check_common(goom_ctx *ctx, int dtype)
{
    if (dtype != GOOM_C64 && dtype != GOOM_C128) return fail(ctx, GOOM_EINVAL, "unknown dtype %d", dtype);
    return GOOM_OK;
}

// Checked after the other arguments, so that argument errors are reported (and can be
// tested) even without a usable device; then makes the context's device current.
static int need_ctx(goom_ctx *ctx)
{
    if (!ctx) return fail(nullptr, GOOM_EINVAL, "null context");
    if (!ctx->prof_keep) prof_reset(ctx); // (an entry point that calls another one keeps the records so far)
    return check_hip(ctx, hipSetDevice(ctx->device), "hipSetDevice");
}

// Chunks per batch item for the three-phase scan: enough chains to fill the chip, but not so many
// that the serial middle phase (one step per chunk) dominates: the serial depth is about
// 2 * chunk_len + chunks, smallest near chunks = sqrt(2 T).  The 128-wide kernel runs one workgroup
// per compute unit and the 64-wide one four, and their chains are long, so a partly filled last round
// of workgroups costs a whole round: there the chain count is one full round (256 or 1024 chains; 512
// for the 64-wide double kernel, which runs two workgroups per compute unit).
static long long default_chunk_len(long long T, long long batch, long long requested, int dp, int dtype)
{
    if (requested > 0) return requested < T ? requested : T;
    const long long slots = dp >= 128 ? 256 : dp >= 64 ? (dtype == GOOM_C128 ? 512 : 1024) : 8192;
    long long c_occ = slots / batch; // never more chains than one round holds
    if (c_occ < 1) c_occ = 1;
    long long c_depth = (long long)std::ceil(std::sqrt(2.0 * (double)T));
    long long c = c_occ < c_depth ? c_occ : c_depth;
    if (c > 1024) c = 1024;
    // Float chains of a few thousand to a few hundred thousand steps, measured (T = 2^11 ... 2^17, chunk lengths
    // 8 ... 512): the square-root rule leaves compute units idle (64 chains at T = 2048), and the grouped carry
    // phase makes many chains cheap; chunks of at least 16 steps (8 at d = 32), 256 chains up to T = 2^14,
    // then 512, and the full round from T = 2^19 (2^16 at d = 32).  Up to twice as fast as the square-root rule
    // at T = 2^11 ... 2^12 and 5 - 20 % above it.
    // The same sweep with double components: chunks of at least 8 steps; 256 chains, from T = 2^14 on 512 at d = 64,
    // from T = 2^13 on 1024 at d = 32 (T = 65 536: 4468 -> 3595 us at d = 64, 1623 -> 862 us at d = 32).
    if (dp == 32 || dp == 64 || dp == 128) {
        long long want;
        if (dp == 128) want = 256;
        else if (dtype == GOOM_C64 && dp == 64) want = T < (1 << 15) ? 256 : T < (1 << 19) ? 512 : 1024;
        else if (dtype == GOOM_C64) want = T < (1 << 14) ? 256 : T < (1 << 16) ? 512 : 1024;
        else if (dp == 64) want = T < (1 << 14) ? 256 : 512;
        else want = T < (1 << 13) ? 256 : 1024;
        const long long shortest = (dtype == GOOM_C64 && dp != 32) ? 16 : 8;
        if (want > T / shortest) want = T / shortest;
        if (want < 1) want = 1;
        c = want < c_occ ? want : c_occ;
    }
    // 16-wide tiles and below: a step is a couple of hundred instructions of one wave and the carry phase is
    // grouped, so what matters is enough chains to give every SIMD several waves (chunks of at least 16 steps;
    // measured at T = 2^22: 8192 chunks beat 1024 by 3.5 x at d = 8 and beat 16384, whose carry phase is longer)
    if (dp <= 16) {
        c = c_occ;
        if (c > T / 16) c = T / 16;
    }
    // the 32-wide double kernel holds six workgroups per compute unit: one full round of 1536 chains when
    // the chunks stay long (measured at T = 2^19: 5.6 ms against 5.9 with 1024 chains and 6.4 with 2048)
    if (dtype == GOOM_C128 && dp == 32 && batch == 1 && T >= 64 * 1536) c = 1536;
    if (c < 1) c = 1;
    long long L = (T + c - 1) / c;
    return L < 1 ? 1 : L;
}

// Layout of one scan in the workspace.
//   totals  : product of every chunk, [batch][C] factored matrices of m_tot columns
//   carries : the prefix that enters every chunk, factored matrices of m_state columns
// The carries are the prefixes of the chunk products, which is a scan again.  With few
// chunks one workgroup per batch item walks them in order.  With many, the same three
// steps are applied once more: chunk products are multiplied down in groups of S (group
// products), one chain walks the G group products, and every group is then re-walked
// from its incoming prefix.  Serial depth falls from C to about 2 S + G steps.  Carries
// of a grouped scan are stored per group with S + 1 entries (the last one repeats the
// first of the next group).
struct ScanPlan {
    long long L, C;  // chunk length, chunks per batch item
    long long nt;    // chunk products the carry phase walks (C - 1 for a scan, C for a reduction)
    long long S, G;  // group size and group count of the carry phase (S = 0: not grouped)
    int dp;
    FactLayout tot, car;
    size_t tot_bytes, car_bytes, gtot_bytes, gcar_bytes;
    size_t total() const { return tot_bytes + car_bytes + gtot_bytes + gcar_bytes; }
};

// fact_dtype: component type of the factored matrices in the workspace when it differs from the GOOMs' (the float
// recurrence keeps its chunk products and carries in double)
static ScanPlan plan_scan(long long T, int d, int m_tot, int m_state, long long batch, int dtype,
                          long long requested_chunk, bool final_only, int fact_dtype = -1)
{
    ScanPlan p;
    if (fact_dtype < 0) fact_dtype = dtype;
    // one tile size for every phase (the factored matrices they hand to each other have that many rows): wide
    // enough for the widest state
    p.dp = chain_padded_dim(d, d, m_tot > m_state ? m_tot : m_state);
    p.L = default_chunk_len(T, batch, requested_chunk, p.dp, dtype);
    p.C = (T + p.L - 1) / p.L;
    p.nt = final_only ? p.C : p.C - 1;
    p.tot = fact_layout(p.dp, m_tot, fact_dtype);
    p.car = fact_layout(p.dp, m_state, fact_dtype);
    p.S = 0;
    p.G = 0;
    if (p.nt > 96) {
        p.S = (long long)std::ceil(std::sqrt((double)p.nt));
        p.G = (p.nt + p.S - 1) / p.S;
    }
    p.tot_bytes = p.C > 1 ? (size_t)batch * p.C * p.tot.stride : 0;
    p.gtot_bytes = p.S ? (size_t)batch * p.G * p.tot.stride : 0;
    p.gcar_bytes = p.S ? (size_t)batch * p.G * p.car.stride : 0;
    if (p.C <= 1 || final_only)
        p.car_bytes = 0;
    else if (p.S)
        p.car_bytes = (size_t)batch * p.G * (p.S + 1) * p.car.stride;
    else
        p.car_bytes = (size_t)batch * p.C * p.car.stride;
    return p;
}

static int check_scan_args(goom_ctx *ctx, const void *M, const void *out, long long T, int d, int m, long long batch,
                           int dtype, const goom_scan_opts *opts, int max_dim = GOOM_MAX_DIM)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (!M || !out) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (T <= 0 || batch <= 0 || d <= 0 || m <= 0) return fail(ctx, GOOM_EINVAL, "sizes must be positive (T=%lld d=%d m=%d batch=%lld)", T, d, m, batch);
    if (d > max_dim || m > max_dim) return fail(ctx, GOOM_EUNSUPPORTED, "d and m must be <= %d (d=%d m=%d)", max_dim, d, m);
    if (opts && opts->flags != 0) return fail(ctx, GOOM_EINVAL, "unknown scan flags 0x%x", opts->flags);
    if (opts && opts->chunk_len < 0) return fail(ctx, GOOM_EINVAL, "negative chunk_len");
    if (!aligned(M, 16) || !aligned(out, 16)) return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    return GOOM_OK;
}

static int check_workspace(goom_ctx *ctx, const void *ws, size_t have, size_t need)
{
    if (need == 0) return GOOM_OK;
    if (!ws) return fail(ctx, GOOM_EWORKSPACE, "workspace of %zu bytes required, none given", need);
    if (have < need) return fail(ctx, GOOM_EWORKSPACE, "workspace too small: %zu bytes given, %zu required", have, need);
    if (!aligned(ws, 256)) return fail(ctx, GOOM_EINVAL, "workspace must be 256-byte aligned");
    return GOOM_OK;
}

// What the carry phase needs to know about the state it carries.
struct CarryState {
    int m;                 // columns of the carried state
    int init_mode;         // 0 identity, 2 GOOM, 3 zero
    const void *init;      // GOOM initial state per batch item (init_mode 2)
    long long init_stride;
    bool bias;             // chunk products are augmented [A | b]: carry a vector, add b
    void *final_goom;      // reduction: the last prefix as GOOMs, [batch, d, m]
};

// Phase 2: prefixes of the chunk products.  On return (for a scan) `carries` holds the
// prefix entering every chunk, indexed as described at ScanPlan.
static int carry_phase(goom_ctx *ctx, const ScanPlan &p, int dtype, int d, long long batch, unsigned char *totals,
                       unsigned char *carries, unsigned char *gtot, unsigned char *gcar, const CarryState &cs,
                       const char *label)
{
    ChainLaunch base;
    std::memset(&base, 0, sizeof base);
    base.dp = p.dp;
    base.dtype = dtype;
    base.n = d;
    base.d = d;
    base.batch = batch;
    base.left_fact = 1;
    base.left_fact_cols = p.tot.cols_padded;
    base.left_step_stride = (long long)p.tot.stride;
    base.label = label;

    if (!p.S) { // one chain per batch item over all chunk products
        ChainLaunch l = base;
        l.m = cs.m;
        l.left = totals;
        l.left_batch_stride = (long long)p.C * p.tot.stride;
        l.steps = p.nt;
        l.chunk_len = p.nt;
        l.chunks_launched = 1;
        l.init_mode = cs.init_mode;
        l.init = cs.init;
        l.init_stride = cs.init_stride;
        l.bias_mode = cs.bias ? 2 : 0;
        l.bias_col = 0;
        if (cs.final_goom) {
            l.out_goom = cs.final_goom;
            l.out_goom_last_only = 1;
        } else {
            l.out_fact_steps = carries;
            l.fact_stride = (long long)p.car.stride;
            l.fact_cols = p.car.cols_padded;
        }
        return launch_chain(ctx, l);
    }
    { // group products (the last group's is needed only by the reduction)
        ChainLaunch l = base;
        l.m = cs.bias ? d + 1 : d;
        l.left = totals;
        l.left_batch_stride = (long long)p.C * p.tot.stride;
        l.steps = p.nt;
        l.chunk_len = p.S;
        l.chunks_launched = cs.final_goom ? p.G : p.G - 1;
        l.init_mode = 0;
        l.bias_mode = cs.bias ? 2 : 0;
        l.bias_col = d;
        l.out_fact_final = gtot;
        l.final_common_exponent = 1;
        l.fact_stride = (long long)p.tot.stride;
        l.fact_cols = p.tot.cols_padded;
        if (int s = launch_chain(ctx, l)) return s;
    }
    { // prefixes of the group products
        ChainLaunch l = base;
        l.m = cs.m;
        l.left = gtot;
        l.left_batch_stride = (long long)p.G * p.tot.stride;
        l.steps = cs.final_goom ? p.G : p.G - 1;
        l.chunk_len = l.steps;
        l.chunks_launched = 1;
        l.init_mode = cs.init_mode;
        l.init = cs.init;
        l.init_stride = cs.init_stride;
        l.bias_mode = cs.bias ? 2 : 0;
        l.bias_col = 0;
        if (cs.final_goom) {
            l.out_goom = cs.final_goom;
            l.out_goom_last_only = 1;
            return launch_chain(ctx, l);
        }
        l.out_fact_steps = gcar;
        l.fact_stride = (long long)p.car.stride;
        l.fact_cols = p.car.cols_padded;
        if (int s = launch_chain(ctx, l)) return s;
    }
    { // every group again, from its incoming prefix: the carries of its chunks
        ChainLaunch l = base;
        l.m = cs.m;
        l.left = totals;
        l.left_batch_stride = (long long)p.C * p.tot.stride;
        l.steps = p.nt;
        l.chunk_len = p.S;
        l.chunks_launched = p.G;
        l.init_mode = 1;
        l.init = gcar;
        l.init_stride = (long long)p.car.stride;
        l.bias_mode = cs.bias ? 2 : 0;
        l.bias_col = 0;
        l.out_fact_steps = carries;
        l.fact_stride = (long long)p.car.stride;
        l.fact_cols = p.car.cols_padded;
        return launch_chain(ctx, l);
    }
}

// scan and reduce share one driver; `final_only` selects the reduction
static int run_scan(goom_ctx *ctx, const void *M, const void *init, void *P, long long T, int d, int m, long long batch,
                    int dtype, const goom_scan_opts *opts, void *ws, size_t ws_bytes, bool final_only, bool left_real = false)
{
    if (int s = check_scan_args(ctx, M, P, T, d, m, batch, dtype, opts, GOOM_MAX_DIM_LMME)) return s;
    if (!init && m != d) return fail(ctx, GOOM_EINVAL, "without an initial state the outputs are d x d (m=%d d=%d)", m, d);
    if (init && !aligned(init, 16)) return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    if (d > GOOM_MAX_DIM || m > GOOM_MAX_DIM) {
        // the state no longer fits a workgroup: chains advance step by step through a tiled GEMM
        const long long req = opts ? opts->chunk_len : 0;
        const bool f32 = dtype == GOOM_C64;
        const size_t need = f32 ? scan_large_workspace_bytes(T, d, m, batch, req, final_only) : scan_large_f64_workspace_bytes(T, d, m, batch, req, final_only);
        if (int s = check_workspace(ctx, ws, ws_bytes, need)) return s;
        if (int s = need_ctx(ctx)) return s;
        return f32 ? run_scan_large(ctx, M, init, P, T, d, m, batch, req, ws, final_only)
                   : run_scan_large_f64(ctx, M, init, P, T, d, m, batch, req, ws, final_only);
    }
    const ScanPlan p = plan_scan(T, d, d, m, batch, dtype, opts ? opts->chunk_len : 0, final_only);
    if (int s = check_workspace(ctx, ws, ws_bytes, p.total())) return s;
    const size_t cb = 2 * comp_bytes(dtype);
    if (int s = need_ctx(ctx)) return s;

    ChainLaunch base;
    std::memset(&base, 0, sizeof base);
    base.dp = p.dp;
    base.dtype = dtype;
    base.n = d;
    base.d = d;
    base.batch = batch;
    base.left = M;
    base.left_real = left_real ? 1 : 0;
    const size_t cbl = left_real ? comp_bytes(dtype) : cb; // bytes per entry of a left factor
    base.left_batch_stride = (long long)T * d * d * cbl;
    base.left_step_stride = (long long)d * d * cbl;
    base.steps = T;

    if (p.C == 1) { // one chain per batch item walks everything
        ChainLaunch l = base;
        l.m = m;
        l.chunk_len = T;
        l.chunks_launched = 1;
        l.init_mode = init ? 2 : 0;
        l.init = init;
        l.init_stride = (long long)d * m * cb;
        l.out_goom = P;
        l.out_goom_last_only = final_only ? 1 : 0;
        l.label = "scan_single_chunk";
        return launch_chain(ctx, l);
    }

    unsigned char *totals = static_cast<unsigned char *>(ws);
    unsigned char *carries = totals + p.tot_bytes;
    unsigned char *gtot = carries + p.car_bytes;
    unsigned char *gcar = gtot + p.gtot_bytes;

    { // phase 1: product of every chunk (the last chunk's is needed only by the reduction)
        ChainLaunch l = base;
        l.m = d;
        l.chunk_len = p.L;
        l.chunks_launched = p.nt;
        l.init_mode = 0;
        l.out_fact_final = totals;
        l.final_common_exponent = 1;
        l.fact_stride = (long long)p.tot.stride;
        l.fact_cols = p.tot.cols_padded;
        l.label = "scan_phase1_chunk_products";
        if (int s = launch_chain(ctx, l)) return s;
    }
    { // phase 2: prefixes of the chunk products
        CarryState cs;
        cs.m = m;
        cs.init_mode = init ? 2 : 0;
        cs.init = init;
        cs.init_stride = (long long)d * m * cb;
        cs.bias = false;
        cs.final_goom = final_only ? P : nullptr;
        if (int s = carry_phase(ctx, p, dtype, d, batch, totals, carries, gtot, gcar, cs, "scan_phase2_carries")) return s;
        if (final_only) return GOOM_OK;
    }
    { // phase 3: every chunk again, from its incoming prefix, writing all outputs
        ChainLaunch l = base;
        l.m = m;
        l.chunk_len = p.L;
        l.chunks_launched = p.C;
        l.init_mode = 1;
        l.init = carries;
        l.init_stride = (long long)p.car.stride;
        l.init_group = p.S;
        l.init_ngroups = p.G;
        l.fact_stride = (long long)p.car.stride;
        l.fact_cols = p.car.cols_padded;
        l.out_goom = P;
        l.label = "scan_phase3_fixup_outputs";
        return launch_chain(ctx, l);
    }
}

// ---- selectively reset scan ------------------------------------------------------------
struct ResetPlan {
    long long L, C;
    int dp;
    FactLayout tot, car;
    size_t tot_bytes, car_bytes, flag_bytes;
    size_t total() const { return tot_bytes + car_bytes + flag_bytes; }
};

// Chunk products, carries and the factorisations at the chunk boundaries are held in double for both formats
// (for complex64 the chain kernels widen every load and round every stored state once): nearly colinear
// columns are exactly what this variant exists for, and their small differences are what a float product loses.
static ResetPlan plan_reset(long long T, int d, long long batch, int dtype, const goom_reset_opts *opts)
{
    ResetPlan p;
    p.L = (opts && opts->chunk_len > 0) ? opts->chunk_len : 128;
    if (p.L > T) p.L = T;
    p.C = (T + p.L - 1) / p.L;
    p.dp = padded_dim(d);
    p.tot = fact_layout(p.dp, d, GOOM_C128);
    p.car = fact_layout(p.dp, d, GOOM_C128);
    p.tot_bytes = (size_t)batch * p.C * p.tot.stride;
    p.car_bytes = (size_t)batch * (p.C + 1) * p.car.stride;
    p.flag_bytes = align_up((size_t)batch * p.C, 256);
    (void)dtype;
    return p;
}

static int run_reset(goom_ctx *ctx, const void *J, const void *S0, void *states, uint8_t *flags, double *growth,
                     double growth_scale, long long T, int d, long long batch, int dtype, const goom_reset_opts *opts,
                     void *ws, size_t ws_bytes)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (!J) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (T <= 0 || batch <= 0 || d <= 0) return fail(ctx, GOOM_EINVAL, "sizes must be positive (T=%lld d=%d batch=%lld)", T, d, batch);
    if (d > GOOM_MAX_DIM) return fail(ctx, GOOM_EUNSUPPORTED, "the reset scan supports d <= %d (d=%d)", GOOM_MAX_DIM, d);
    if (opts && opts->chunk_len < 0) return fail(ctx, GOOM_EINVAL, "negative chunk_len");
    const int policy = opts ? opts->policy : GOOM_RESET_ALWAYS;
    if (policy < GOOM_RESET_NEVER || policy > GOOM_RESET_ALWAYS) return fail(ctx, GOOM_EINVAL, "unknown reset policy %d", policy);
    if (!aligned(J, 16) || (S0 && !aligned(S0, 16)) || (states && !aligned(states, 16)))
        return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    if (growth && !aligned(growth, 8)) return fail(ctx, GOOM_EINVAL, "growth must be 8-byte aligned");
    const ResetPlan p = plan_reset(T, d, batch, dtype, opts);
    if (int s = check_workspace(ctx, ws, ws_bytes, p.total())) return s;
    if (int s = need_ctx(ctx)) return s;
    const size_t cb = 2 * comp_bytes(dtype);
    unsigned char *totals = static_cast<unsigned char *>(ws);
    unsigned char *carries = totals + p.tot_bytes;
    unsigned char *chunk_flags = carries + p.car_bytes;

    ChainLaunch base;
    std::memset(&base, 0, sizeof base);
    base.dp = p.dp;
    base.dtype = GOOM_C128; // double running product
    base.io_c64 = dtype == GOOM_C64 ? 1 : 0;
    base.n = d;
    base.d = d;
    base.m = d;
    base.batch = batch;
    base.left = J;
    base.left_batch_stride = (long long)T * d * d * cb;
    base.left_step_stride = (long long)d * d * cb;
    base.steps = T;
    base.chunk_len = p.L;
    base.chunks_launched = p.C;
    { // phase 1: product of every chunk
        ChainLaunch l = base;
        l.init_mode = 0;
        l.out_fact_final = totals;
        l.final_common_exponent = 1;
        l.fact_stride = (long long)p.tot.stride;
        l.fact_cols = p.tot.cols_padded;
        l.label = "reset_phase1_chunk_products";
        if (int s = launch_chain(ctx, l)) return s;
    }
    ResetLaunch r;
    std::memset(&r, 0, sizeof r);
    r.dtype = dtype;
    r.totals = totals;
    r.tot_stride = (long long)p.tot.stride;
    r.tot_cols = p.tot.cols_padded;
    r.carries = carries;
    r.car_stride = (long long)p.car.stride;
    r.car_cols = p.car.cols_padded;
    r.s0 = S0;
    r.post_states = states;
    r.chunk_flags = chunk_flags;
    r.flags = flags;
    r.growth = growth;
    r.growth_scale = growth_scale;
    r.T = T;
    r.L = p.L;
    r.C = p.C;
    r.batch = batch;
    r.d = d;
    r.policy = policy;
    r.cos_threshold = opts ? opts->cos_threshold : 0.99f;
    // phase 2: prefixes at the chunk boundaries, examined and reset in order
    if (int s = launch_reset_carry(ctx, r)) return s;
    if (states) { // phase 3: every chunk again from its incoming prefix, all states stored
        ChainLaunch l = base;
        l.init_mode = 1;
        l.init = carries;
        l.init_stride = (long long)p.car.stride;
        l.init_group = p.C; // carries hold C + 1 entries per batch item
        l.init_ngroups = 1;
        l.fact_stride = (long long)p.car.stride;
        l.fact_cols = p.car.cols_padded;
        l.out_goom = states;
        l.label = "reset_phase3_states";
        if (int s = launch_chain(ctx, l)) return s;
    }
    if (states || flags) return launch_reset_post(ctx, r);
    return GOOM_OK;
}

} // namespace goom

using namespace goom;

extern "C" {

int goom_version(void) { return GOOM_VERSION; }

const char *goom_status_name(int status)
{
    switch (status) {
    case GOOM_OK: return "GOOM_OK";
    case GOOM_EINVAL: return "GOOM_EINVAL";
    case GOOM_EUNSUPPORTED: return "GOOM_EUNSUPPORTED";
    case GOOM_EWORKSPACE: return "GOOM_EWORKSPACE";
    case GOOM_EHIP: return "GOOM_EHIP";
    case GOOM_ENOMEM: return "GOOM_ENOMEM";
    default: return "GOOM_E?";
    }
}

const char *goom_last_error(const goom_ctx *ctx) { return ctx ? ctx->last_error.c_str() : thread_error(); }

int goom_create(goom_ctx **out, int device, void *stream)
{
    if (!out) return fail(nullptr, GOOM_EINVAL, "null context pointer");
    *out = nullptr;
    if (device < 0) return fail(nullptr, GOOM_EINVAL, "negative device index");
    int count = 0;
    hipError_t e = hipGetDeviceCount(&count);
    if (e != hipSuccess || count <= 0) return fail(nullptr, GOOM_EHIP, "no HIP device available (%s)", hipGetErrorString(e));
    if (device >= count) return fail(nullptr, GOOM_EINVAL, "device %d out of range (%d devices)", device, count);
    hipDeviceProp_t prop;
    if (int s = check_hip(nullptr, hipGetDeviceProperties(&prop, device), "hipGetDeviceProperties")) return s;
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(nullptr, GOOM_EUNSUPPORTED, "device %d is %s; this library is built for gfx950", device, prop.gcnArchName);
    goom_ctx *ctx = new (std::nothrow) goom_ctx;
    if (!ctx) return fail(nullptr, GOOM_ENOMEM, "out of host memory");
    ctx->device = device;
    ctx->stream = static_cast<hipStream_t>(stream);
    resolve_scratch(ctx); // a failure is kept in the context and reported by goom_scan_static
    *out = ctx;
    return GOOM_OK;
}

int goom_destroy(goom_ctx *ctx)
{
    if (!ctx) return GOOM_OK;
    prof_reset(ctx);
    for (auto &r : ctx->prof_pool) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    delete ctx;
    return GOOM_OK;
}

int goom_profile_enable(goom_ctx *ctx, int enable)
{
    if (!ctx) return fail(nullptr, GOOM_EINVAL, "null context");
    ctx->profile = enable != 0;
    return GOOM_OK;
}

int goom_profile_count(const goom_ctx *ctx) { return ctx ? (int)ctx->prof.size() : 0; }

int goom_profile_get(goom_ctx *ctx, int i, const char **label, float *milliseconds)
{
    if (!ctx) return fail(nullptr, GOOM_EINVAL, "null context");
    if (i < 0 || i >= (int)ctx->prof.size()) return fail(ctx, GOOM_EINVAL, "no profiling record %d", i);
    goom_prof_rec &r = ctx->prof[i];
    if (int s = check_hip(ctx, hipEventSynchronize(r.stop), "hipEventSynchronize")) return s;
    float ms = 0.f;
    if (int s = check_hip(ctx, hipEventElapsedTime(&ms, r.start, r.stop), "hipEventElapsedTime")) return s;
    if (label) *label = r.label;
    if (milliseconds) *milliseconds = ms;
    return GOOM_OK;
}

int goom_set_stream(goom_ctx *ctx, void *stream)
{
    if (!ctx) return fail(nullptr, GOOM_EINVAL, "null context");
    ctx->stream = static_cast<hipStream_t>(stream);
    return GOOM_OK;
}

int goom_probe_bandwidth(goom_ctx *ctx, const void *a, void *b, size_t bytes, int mode)
{
    if (mode != GOOM_PROBE_READ && mode != GOOM_PROBE_WRITE && mode != GOOM_PROBE_COPY) return fail(ctx, GOOM_EINVAL, "unknown probe mode %d", mode);
    if (!b || (!a && mode != GOOM_PROBE_WRITE)) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (bytes == 0 || bytes % 16 != 0 || !aligned(b, 16) || (a && !aligned(a, 16)))
        return fail(ctx, GOOM_EINVAL, "the probe wants 16-byte aligned buffers of a multiple of 16 bytes");
    if (int s = need_ctx(ctx)) return s;
    return launch_probe(ctx, a, b, bytes, mode);
}

int goom_probe_matrix_unit(goom_ctx *ctx, void *sink, int64_t iters, int dtype)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (!sink || !aligned(sink, 4)) return fail(ctx, GOOM_EINVAL, "the probe wants 4 bytes of device memory");
    if (iters <= 0 || iters > (1LL << 24)) return fail(ctx, GOOM_EINVAL, "iters must be in 1 ... 2^24 (%lld)", (long long)iters);
    if (int s = need_ctx(ctx)) return s;
    return launch_matrix_probe(ctx, sink, iters, dtype);
}

int goom_to_goom(goom_ctx *ctx, const void *x, void *y, size_t n, int dtype, uint32_t flags)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (flags & ~GOOM_ZERO_FLOOR) return fail(ctx, GOOM_EINVAL, "unknown codec flags 0x%x", flags);
    if (n == 0) return GOOM_OK;
    if (!x || !y) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (!aligned(x, 16) || !aligned(y, 16)) return fail(ctx, GOOM_EINVAL, "codec arrays must be 16-byte aligned");
    if (int s = need_ctx(ctx)) return s;
    return launch_to_goom(ctx, x, y, n, dtype, flags);
}

int goom_from_goom(goom_ctx *ctx, const void *y, void *x, size_t n, int dtype)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (n == 0) return GOOM_OK;
    if (!x || !y) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (!aligned(x, 16) || !aligned(y, 16)) return fail(ctx, GOOM_EINVAL, "codec arrays must be 16-byte aligned");
    if (int s = need_ctx(ctx)) return s;
    return launch_from_goom(ctx, y, x, n, dtype);
}

static bool lmme_is_large(int n, int d, int m) { return n > GOOM_MAX_DIM || d > GOOM_MAX_DIM || m > GOOM_MAX_DIM; }

// 128 x 128 x 128 products with the repair pass: room for the product's row and column shifts, which spares the repair
// pass its own pass over the operands (optional: without it the repair pass takes the maxima itself)
static size_t lmme128_shift_bytes(int64_t batch, int dtype) { return (size_t)batch * 256 * (dtype == GOOM_C64 ? 4 : 8); }

size_t goom_lmme_workspace_bytes(int64_t batch, int n, int d, int m, int dtype, uint32_t flags)
{
    if (batch <= 0 || n <= 0 || d <= 0 || m <= 0 || (dtype != GOOM_C64 && dtype != GOOM_C128)) return 0;
    if (n == 128 && d == 128 && m == 128 && (flags & GOOM_LMME_EXACT)) return lmme128_shift_bytes(batch, dtype);
    if (lmme_tall_applies(n, d, m, dtype)) return 0;
    if (!lmme_is_large(n, d, m)) return 0;
    if (n > GOOM_MAX_DIM_LMME || d > GOOM_MAX_DIM_LMME || m > GOOM_MAX_DIM_LMME) return 0;
    return dtype == GOOM_C64 ? lmme_large_workspace_bytes(batch, n, d, m) : lmme_large_f64_workspace_bytes(batch, n, d, m);
}

int goom_lmme(goom_ctx *ctx, const void *A, const void *B, void *C, int64_t batch, int n, int d, int m, int dtype,
              uint32_t flags, void *workspace, size_t workspace_bytes)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (flags & ~GOOM_LMME_EXACT) return fail(ctx, GOOM_EINVAL, "unknown LMME flags 0x%x", flags);
    if (!A || !B || !C) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (batch <= 0 || n <= 0 || d <= 0 || m <= 0) return fail(ctx, GOOM_EINVAL, "sizes must be positive");
    if (n > GOOM_MAX_DIM_LMME || d > GOOM_MAX_DIM_LMME || m > GOOM_MAX_DIM_LMME)
        return fail(ctx, GOOM_EUNSUPPORTED, "n, d, m must be <= %d", GOOM_MAX_DIM_LMME);
    if (!aligned(A, 16) || !aligned(B, 16) || !aligned(C, 16)) return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    if (lmme_tall_applies(n, d, m, dtype)) {
        // many rows against a small right operand (the input term of the state-space layer): rows streamed past B~ in registers
        if (int s = need_ctx(ctx)) return s;
        if (int s = launch_lmme_tall(ctx, A, B, C, batch, n, d, m)) return s;
        if (flags & GOOM_LMME_EXACT) return launch_lmme_exact(ctx, A, B, C, batch, n, d, m, dtype);
        return GOOM_OK;
    }
    if (lmme_is_large(n, d, m)) {
        // beyond the register-resident kernels: scaled operands, a tiled GEMM and a store pass, through the workspace
        const bool f32 = dtype == GOOM_C64;
        const size_t need = f32 ? lmme_large_workspace_bytes(batch, n, d, m) : lmme_large_f64_workspace_bytes(batch, n, d, m);
        if (int s = check_workspace(ctx, workspace, workspace_bytes, need)) return s;
        if (int s = need_ctx(ctx)) return s;
        if (int s = f32 ? launch_lmme_large(ctx, A, B, C, batch, n, d, m, workspace) : launch_lmme_large_f64(ctx, A, B, C, batch, n, d, m, workspace))
            return s;
        if (flags & GOOM_LMME_EXACT) return launch_lmme_exact(ctx, A, B, C, batch, n, d, m, dtype);
        return GOOM_OK;
    }
    if (int s = need_ctx(ctx)) return s;
    if (n == 128 && d == 128 && m == 128) {
        // the full-size product has a kernel of its own (inner index in tiles, running rescale)
        void *shifts = nullptr;
        if ((flags & GOOM_LMME_EXACT) && workspace && aligned(workspace, 16) && workspace_bytes >= lmme128_shift_bytes(batch, dtype))
            shifts = workspace;
        if (int s = launch_lmme128(ctx, A, B, C, batch, dtype, shifts)) return s;
        if (flags & GOOM_LMME_EXACT) return launch_lmme_exact(ctx, A, B, C, batch, n, d, m, dtype, shifts);
        return GOOM_OK;
    }
    const size_t cb = 2 * (dtype == GOOM_C64 ? 4 : 8);
    ChainLaunch l;
    std::memset(&l, 0, sizeof l);
    l.dtype = dtype;
    l.n = n;
    l.d = d;
    l.m = m;
    l.left = A;
    l.left_batch_stride = (long long)n * d * cb;
    l.left_step_stride = (long long)n * d * cb;
    l.steps = 1;
    l.chunk_len = 1;
    l.chunks_launched = 1;
    l.batch = batch;
    l.init_mode = 2;
    l.init = B;
    l.init_stride = (long long)d * m * cb;
    l.out_goom = C;
    l.label = "lmme";
    if (int s = launch_chain(ctx, l)) return s;
    if (flags & GOOM_LMME_EXACT) return launch_lmme_exact(ctx, A, B, C, batch, n, d, m, dtype);
    return GOOM_OK;
}

size_t goom_scan_workspace_bytes(int64_t T, int d, int m, int64_t batch, int dtype, const goom_scan_opts *opts)
{
    if (T <= 0 || d <= 0 || m <= 0 || batch <= 0 || d > GOOM_MAX_DIM_LMME || m > GOOM_MAX_DIM_LMME) return 0;
    if (dtype != GOOM_C64 && dtype != GOOM_C128) return 0;
    if (d > GOOM_MAX_DIM || m > GOOM_MAX_DIM)
        return dtype == GOOM_C64 ? scan_large_workspace_bytes(T, d, m, batch, opts ? opts->chunk_len : 0, false)
                                 : scan_large_f64_workspace_bytes(T, d, m, batch, opts ? opts->chunk_len : 0, false);
    ScanPlan p = plan_scan(T, d, d, m, batch, dtype, opts ? opts->chunk_len : 0, false);
    return p.total();
}

size_t goom_reduce_workspace_bytes(int64_t T, int d, int m, int64_t batch, int dtype, const goom_scan_opts *opts)
{
    if (T <= 0 || d <= 0 || m <= 0 || batch <= 0 || d > GOOM_MAX_DIM_LMME || m > GOOM_MAX_DIM_LMME) return 0;
    if (dtype != GOOM_C64 && dtype != GOOM_C128) return 0;
    if (d > GOOM_MAX_DIM || m > GOOM_MAX_DIM)
        return dtype == GOOM_C64 ? scan_large_workspace_bytes(T, d, m, batch, opts ? opts->chunk_len : 0, true)
                                 : scan_large_f64_workspace_bytes(T, d, m, batch, opts ? opts->chunk_len : 0, true);
    ScanPlan p = plan_scan(T, d, d, m, batch, dtype, opts ? opts->chunk_len : 0, true);
    return p.total();
}

int goom_scan(goom_ctx *ctx, const void *M, const void *init, void *P, int64_t T, int d, int m, int64_t batch, int dtype,
              const goom_scan_opts *opts, void *workspace, size_t workspace_bytes)
{
    return run_scan(ctx, M, init, P, T, d, m, batch, dtype, opts, workspace, workspace_bytes, false);
}

int goom_scan_static(goom_ctx *ctx, const void *M, const void *init, void *P, int64_t T, int d, int m, int64_t batch, int dtype,
                     const goom_scan_opts *opts)
{
    // argument errors first (reported without a device); the size check uses the same plan as goom_scan
    if (int s = check_scan_args(ctx, M, P, T, d, m, batch, dtype, opts, GOOM_MAX_DIM_LMME)) return s;
    goom_scan_opts eff = opts ? *opts : goom_scan_opts{0, 0};
    size_t need = goom_scan_workspace_bytes(T, d, m, batch, dtype, &eff);
    if (need > (size_t)GOOM_STATIC_SCRATCH_BYTES && eff.chunk_len == 0) {
        // the default plan has more chunks than the array holds products of: the shortest chunks, by powers of two,
        // that fit (fewer chunks, a smaller workspace; the result is the same scan)
        for (long long L = 8; L < T; L *= 2) {
            goom_scan_opts longer = eff;
            longer.chunk_len = L;
            const size_t n = goom_scan_workspace_bytes(T, d, m, batch, dtype, &longer);
            if (n > 0 && n <= (size_t)GOOM_STATIC_SCRATCH_BYTES) {
                eff = longer;
                need = n;
                break;
            }
        }
    }
    if (need > (size_t)GOOM_STATIC_SCRATCH_BYTES)
        return fail(ctx, GOOM_EWORKSPACE, "this scan needs %zu bytes of scratch memory; goom_scan_static holds %zu (use goom_scan with a workspace)",
                    need, (size_t)GOOM_STATIC_SCRATCH_BYTES);
    if (!ctx) return fail(nullptr, GOOM_EINVAL, "null context");
    if (!ctx->scratch) return fail(ctx, GOOM_EHIP, "%s", ctx->scratch_error.empty() ? "static scratch memory unavailable" : ctx->scratch_error.c_str());
    // nothing in the workspace has to start at zero: every phase writes what the next one reads
    return run_scan(ctx, M, init, P, T, d, m, batch, dtype, &eff, ctx->scratch, (size_t)GOOM_STATIC_SCRATCH_BYTES, false);
}

int goom_reduce(goom_ctx *ctx, const void *M, const void *init, void *P_final, int64_t T, int d, int m, int64_t batch,
                int dtype, const goom_scan_opts *opts, void *workspace, size_t workspace_bytes)
{
    return run_scan(ctx, M, init, P_final, T, d, m, batch, dtype, opts, workspace, workspace_bytes, true);
}

// Scans of real matrices: the hot float kernel reads them directly where it applies; elsewhere they are
// encoded into the workspace first.
static bool real_input_native(int d, int m, int dtype) { return dtype == GOOM_C64 && m == d && (d == 32 || d == 64 || d == 128); }

static size_t real_scan_workspace(int64_t T, int d, int m, int64_t batch, int dtype, const goom_scan_opts *opts, bool final_only)
{
    const size_t base = final_only ? goom_reduce_workspace_bytes(T, d, m, batch, dtype, opts) : goom_scan_workspace_bytes(T, d, m, batch, dtype, opts);
    if (T <= 0 || d <= 0 || m <= 0 || batch <= 0 || (dtype != GOOM_C64 && dtype != GOOM_C128)) return 0;
    if (real_input_native(d, m, dtype)) return base;
    return align_up(base, 256) + align_up((size_t)batch * (size_t)T * d * d * 2 * comp_bytes(dtype), 256);
}

static int run_scan_real(goom_ctx *ctx, const void *X, const void *init, void *P, long long T, int d, int m, long long batch, int dtype,
                         const goom_scan_opts *opts, void *ws, size_t ws_bytes, bool final_only)
{
    if (int s = check_scan_args(ctx, X, P, T, d, m, batch, dtype, opts, GOOM_MAX_DIM_LMME)) return s;
    if (real_input_native(d, m, dtype)) return run_scan(ctx, X, init, P, T, d, m, batch, dtype, opts, ws, ws_bytes, final_only, true);
    const size_t base = final_only ? goom_reduce_workspace_bytes(T, d, m, batch, dtype, opts) : goom_scan_workspace_bytes(T, d, m, batch, dtype, opts);
    const size_t zoff = align_up(base, 256);
    const size_t need = zoff + align_up((size_t)batch * (size_t)T * d * d * 2 * comp_bytes(dtype), 256);
    if (int s = check_workspace(ctx, ws, ws_bytes, need)) return s;
    if (int s = need_ctx(ctx)) return s;
    void *Z = static_cast<unsigned char *>(ws) + zoff;
    if (int s = launch_to_goom(ctx, X, Z, (size_t)batch * (size_t)T * d * d, dtype, 0)) return s;
    return run_scan(ctx, Z, init, P, T, d, m, batch, dtype, opts, base ? ws : nullptr, base, final_only, false);
}

size_t goom_scan_real_workspace_bytes(int64_t T, int d, int m, int64_t batch, int dtype, const goom_scan_opts *opts)
{
    return real_scan_workspace(T, d, m, batch, dtype, opts, false);
}

size_t goom_reduce_real_workspace_bytes(int64_t T, int d, int m, int64_t batch, int dtype, const goom_scan_opts *opts)
{
    return real_scan_workspace(T, d, m, batch, dtype, opts, true);
}

int goom_scan_real(goom_ctx *ctx, const void *X, const void *init, void *P, int64_t T, int d, int m, int64_t batch, int dtype,
                   const goom_scan_opts *opts, void *workspace, size_t workspace_bytes)
{
    return run_scan_real(ctx, X, init, P, T, d, m, batch, dtype, opts, workspace, workspace_bytes, false);
}

int goom_reduce_real(goom_ctx *ctx, const void *X, const void *init, void *P_final, int64_t T, int d, int m, int64_t batch, int dtype,
                     const goom_scan_opts *opts, void *workspace, size_t workspace_bytes)
{
    return run_scan_real(ctx, X, init, P_final, T, d, m, batch, dtype, opts, workspace, workspace_bytes, true);
}

// The float recurrence with d = 16 or 32 keeps its chunk products and carries in double: a float product of many
// matrices carries its rounding error relative to its norm, and applied to a carried vector that lies nearly
// orthogonal to the product's dominant input direction that error has no bound relative to the result.
struct AffinePlan {
    ScanPlan p;
    bool f64;        // chunk products and carries in double (float GOOMs in and out)
    size_t h0_bytes; // room for an initial state widened to double components
    size_t total() const { return align_up(p.total(), 256) + h0_bytes; }
};

static AffinePlan plan_affine(long long T, int d, long long batch, int dtype, const goom_scan_opts *opts)
{
    AffinePlan ap;
    const long long req = opts ? opts->chunk_len : 0;
    ap.p = plan_scan(T, d, d + 1, 1, batch, dtype, req, false);
    ap.f64 = dtype == GOOM_C64 && (d == 16 || d == 32) && ap.p.dp == d && ap.p.C > 1;
    ap.h0_bytes = 0;
    if (ap.f64) {
        ap.p = plan_scan(T, d, d + 1, 1, batch, dtype, req, false, GOOM_C128);
        ap.h0_bytes = align_up((size_t)batch * d * 16, 256);
    }
    return ap;
}

// Batches of many sequences with a matrix per step (float components, d = 32, default chunking): each sequence is walked start
// to end by one workgroup, which takes about 0.27 us a step whatever the batch (up to one workgroup per compute unit); the chunked
// scan takes about 3.8 ns a token, so the walk wins from about 75 sequences on.
constexpr long long kAffineSequentialMinBatch = 96;
static bool affine_sequential_applies(long long T, int d, long long batch, int dtype, const goom_scan_opts *opts)
{
    const bool ti = opts && (opts->flags & GOOM_AFFINE_TIME_INVARIANT);
    return dtype == GOOM_C64 && d == 32 && !ti && (!opts || opts->chunk_len == 0) && batch >= kAffineSequentialMinBatch && T >= 1;
}

size_t goom_affine_scan_workspace_bytes(int64_t T, int d, int64_t batch, int dtype, const goom_scan_opts *opts)
{
    if (T <= 0 || d <= 0 || batch <= 0 || d > GOOM_MAX_DIM) return 0;
    if (dtype != GOOM_C64 && dtype != GOOM_C128) return 0;
    return plan_affine(T, d, batch, dtype, opts).total();
}

// Scaled states (Section 4.3, eq. 27) come straight out of the matrix-vector walk where that kernel serves the
// last phase; otherwise the states are written as GOOMs to the workspace and converted.
// the scaled states are written by the matrix-vector walk itself
static bool affine_scaled_is_fused(const ScanPlan &p, int d, int dtype) { return dtype == GOOM_C64 && (d == 16 || d == 32 || d == 64) && p.C > 1; }

static size_t affine_states_bytes(long long T, int d, long long batch, int dtype)
{
    return align_up((size_t)batch * (size_t)T * (size_t)d * 2 * comp_bytes(dtype), 256);
}

size_t goom_affine_scan_scaled_workspace_bytes(int64_t T, int d, int64_t batch, int dtype, const goom_scan_opts *opts)
{
    if (T <= 0 || d <= 0 || batch <= 0 || d > GOOM_MAX_DIM) return 0;
    if (dtype != GOOM_C64 && dtype != GOOM_C128) return 0;
    const AffinePlan ap = plan_affine(T, d, batch, dtype, opts);
    return align_up(ap.total(), 256) + (affine_scaled_is_fused(ap.p, d, dtype) ? 0 : affine_states_bytes(T, d, batch, dtype));
}

// adjoint_shift: NULL, or [batch, T] floats: the recurrence then runs on the transposes of A's matrices in reverse
// order, the log-magnitudes of step s's factor shifted by adjoint_shift[s] (the backward pass; float GOOMs with the
// double chunk products only).
static int run_affine(goom_ctx *ctx, const void *A, const void *bias, const void *h0, void *H, void *scaled, void *logscale,
                      int64_t T, int d, int64_t batch, int dtype, const goom_scan_opts *opts, void *ws, size_t ws_bytes,
                      const float *adjoint_shift = nullptr, const float *io_shift = nullptr)
{
    // io_shift: [batch, T] whole numbers c_s; the bias enters as bias[s] e^(-c_s), the states leave as h_s e^(c_s) (the adjoint
    // recurrence over one matrix)
    // adjoint_shift: the adjoint recurrence, read from the forward pass's matrices (transposed, in reverse order, shifted);
    goom_scan_opts plain = opts ? *opts : goom_scan_opts{0, 0};
    const bool ti = (plain.flags & GOOM_AFFINE_TIME_INVARIANT) != 0;
    plain.flags &= ~GOOM_AFFINE_TIME_INVARIANT;
    const bool want_scaled = H == nullptr;
    if (int s = check_scan_args(ctx, A, want_scaled ? scaled : H, T, d, 1, batch, dtype, &plain)) return s;
    if (!bias) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (d > GOOM_MAX_DIM) return fail(ctx, GOOM_EUNSUPPORTED, "the recurrence with bias needs d <= %d", GOOM_MAX_DIM);
    if (!aligned(bias, 16) || (h0 && !aligned(h0, 16))) return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    if (logscale && !aligned(logscale, comp_bytes(dtype))) return fail(ctx, GOOM_EINVAL, "misaligned data pointer");
    const AffinePlan ap = plan_affine(T, d, batch, dtype, opts);
    const ScanPlan &p = ap.p;
    const bool fused = want_scaled && affine_scaled_is_fused(p, d, dtype);
    const size_t need = want_scaled ? align_up(ap.total(), 256) + (fused ? 0 : affine_states_bytes(T, d, batch, dtype)) : ap.total();
    if (int s = check_workspace(ctx, ws, ws_bytes, need)) return s;
    if (int s = need_ctx(ctx)) return s;
    if (affine_sequential_applies(T, d, batch, dtype, opts) && !io_shift)
        // enough sequences to fill the chip one workgroup each: no chunks, every matrix read once
        return goom_chain::launch_affine_seq(ctx, A, bias, h0, H, want_scaled ? scaled : nullptr, want_scaled ? logscale : nullptr, T, batch,
                                             adjoint_shift);
    const size_t cb = 2 * comp_bytes(dtype);
    if (want_scaled && !fused) {
        // the states as GOOMs behind the scan's own workspace, then their scaled exponentials
        H = static_cast<unsigned char *>(ws) + align_up(ap.total(), 256);
        if (int s = run_affine(ctx, A, bias, h0, H, nullptr, nullptr, T, d, batch, dtype, opts, ws, ap.total())) return s;
        return launch_scaled_exp(ctx, H, scaled, logscale, (size_t)batch * (size_t)T, d, dtype);
    }
    const int f64 = ap.f64 ? 1 : 0;
    if (adjoint_shift && (!f64 || ti || want_scaled)) return fail(ctx, GOOM_EUNSUPPORTED, "transposed factors in reverse order: float GOOMs, d = 16 or 32, several chunks");

    ChainLaunch base;
    std::memset(&base, 0, sizeof base);
    base.dtype = dtype;
    base.n = d;
    base.d = d;
    base.batch = batch;
    base.left = A;
    base.left_batch_stride = ti ? (long long)d * d * cb : (long long)T * d * d * cb;
    base.left_step_stride = ti ? 0 : (long long)d * d * cb; // a time-invariant matrix is every step's factor
    base.steps = T;
    base.bias_mode = 1;
    base.bias = bias;
    base.left_shift = adjoint_shift;
    base.io_shift = io_shift;
    if (io_shift && !(ti && !want_scaled)) return fail(ctx, GOOM_EUNSUPPORTED, "rescaled bias and states: one matrix for all steps, GOOM states");

    if (p.C == 1) {
        ChainLaunch l = base;
        l.m = 1;
        l.bias_col = 0;
        l.chunk_len = T;
        l.chunks_launched = 1;
        l.init_mode = h0 ? 2 : 3;
        l.init = h0;
        l.init_stride = (long long)d * cb;
        l.out_goom = H;
        l.label = "affine_single_chunk";
        return launch_chain(ctx, l);
    }
    unsigned char *totals = static_cast<unsigned char *>(ws);
    unsigned char *carries = totals + p.tot_bytes;
    unsigned char *gtot = carries + p.car_bytes;
    unsigned char *gcar = gtot + p.gtot_bytes;
    if (ti && dtype == GOOM_C64 && (d == 16 || d == 32 || d == 64)) {
        // phase 1, time-invariant: every chunk's total is [A^L | b*_c].  A^L once per batch item (a chain
        // of L equal factors), copied to all chunks; b*_c by a matrix-vector walk of the chunk from zero.
        ChainLaunch l = base;
        l.bias_mode = 0;
        l.bias = nullptr;
        l.io_shift = nullptr;
        l.m = d;
        l.steps = p.L;
        l.chunk_len = p.L;
        l.chunks_launched = 1;
        l.init_mode = 0;
        l.out_fact_final = totals;
        l.final_common_exponent = 1;
        l.fact_stride = (long long)p.tot.stride * p.C;
        l.fact_cols = p.tot.cols_padded;
        l.label = "affine_phase1_matrix_power";
        if (f64) { // the double-state chunk kernel with no bias: [A^L | 0]
            l.acc_f64 = 1;
            l.m = d + 1;
            l.bias_col = d;
        }
        // A^L = (A^L1)^L2 shortens the chain of dependent products from L to L1 + L2 (one wave-sized chain per batch item: its
        // length is the whole cost).  The inner power goes to the second chunk's slot, which is overwritten afterwards.
        const long long L1 = (p.L >= 64 && p.L % 16 == 0) ? (p.L >= 1024 && p.L % 32 == 0 ? 32 : 16) : 0;
        if (L1) {
            l.steps = L1;
            l.chunk_len = L1;
            l.out_fact_final = totals + p.tot.stride;
        }
        if (int s = launch_chain(ctx, l)) return s;
        if (L1) { // the outer power: L2 equal factored factors, as the carry phase multiplies chunk products
            ChainLaunch o;
            std::memset(&o, 0, sizeof o);
            o.dp = p.dp;
            o.dtype = f64 ? GOOM_C128 : dtype;
            o.n = d;
            o.d = d;
            o.m = f64 ? d + 1 : d; // (the double chunk kernel wrote a zero bias column, the float one none)
            o.batch = batch;
            o.left_fact = 1;
            o.left_fact_cols = p.tot.cols_padded;
            o.left = totals + p.tot.stride;
            o.left_batch_stride = (long long)p.tot.stride * p.C;
            o.left_step_stride = 0; // the same factor at every step
            o.steps = p.L / L1;
            o.chunk_len = o.steps;
            o.chunks_launched = 1;
            o.init_mode = 0;
            o.bias_mode = f64 ? 2 : 0; // (the factor's bias column is zero, and stays so)
            o.bias_col = d;
            o.out_fact_final = totals;
            o.final_common_exponent = 1;
            o.fact_stride = (long long)p.tot.stride * p.C;
            o.fact_cols = p.tot.cols_padded;
            o.label = "affine_phase1_matrix_power";
            if (int s = launch_chain(ctx, o)) return s;
        }
        if (int s = goom_chain::launch_replicate_power(ctx, totals, (long long)p.tot.stride, p.tot.cols_padded, p.dp, d, batch, p.C - 1, p.C, f64 != 0)) return s;
        ChainLaunch w = base;
        w.m = 1;
        w.bias_col = d;
        w.chunk_len = p.L;
        w.chunks_launched = p.C - 1;
        w.init_mode = 3;
        w.out_fact_final = totals;
        w.fact_stride = (long long)p.tot.stride;
        w.fact_cols = p.tot.cols_padded;
        w.fact_f64 = f64;
        w.label = "affine_phase1_chunk_vectors";
        if (int s = launch_chain(ctx, w)) return s;
    } else { // phase 1: augmented chunk products [A* | b*]
        ChainLaunch l = base;
        l.m = d + 1;
        l.bias_col = d;
        l.chunk_len = p.L;
        l.chunks_launched = p.C - 1;
        l.init_mode = 0;
        l.out_fact_final = totals;
        l.final_common_exponent = 1;
        l.fact_stride = (long long)p.tot.stride;
        l.fact_cols = p.tot.cols_padded;
        l.acc_f64 = f64;
        l.label = "affine_phase1_chunk_products";
        if (int s = launch_chain(ctx, l)) return s;
    }
    { // phase 2: h at the chunk boundaries
        CarryState cs;
        cs.m = 1;
        cs.init_mode = h0 ? 2 : 3;
        cs.init = h0;
        cs.init_stride = (long long)d * cb;
        cs.bias = true;
        cs.final_goom = nullptr;
        if (f64 && h0) { // the double carry kernels read the initial state with double components
            void *h0w = static_cast<unsigned char *>(ws) + align_up(p.total(), 256);
            if (int s = launch_widen_goom(ctx, h0, h0w, (size_t)batch * d)) return s;
            cs.init = h0w;
            cs.init_stride = (long long)d * 16;
        }
        if (int s = carry_phase(ctx, p, f64 ? GOOM_C128 : dtype, d, batch, totals, carries, gtot, gcar, cs, "affine_phase2_carries")) return s;
    }
    { // phase 3: matrix-vector walk of every chunk
        ChainLaunch l = base;
        l.m = 1;
        l.bias_col = 0;
        l.chunk_len = p.L;
        l.chunks_launched = p.C;
        l.init_mode = 1;
        l.init = carries;
        l.init_stride = (long long)p.car.stride;
        l.init_group = p.S;
        l.init_ngroups = p.G;
        l.fact_stride = (long long)p.car.stride;
        l.fact_cols = p.car.cols_padded;
        l.out_goom = H;
        l.out_scaled = fused ? scaled : nullptr;
        l.out_logscale = fused ? logscale : nullptr;
        l.fact_f64 = f64;
        l.label = "affine_phase3_outputs";
        return launch_chain(ctx, l);
    }
}

int goom_affine_scan(goom_ctx *ctx, const void *A, const void *bias, const void *h0, void *H, int64_t T, int d,
                     int64_t batch, int dtype, const goom_scan_opts *opts, void *ws, size_t ws_bytes)
{
    if (!H) return fail(ctx, GOOM_EINVAL, "null data pointer");
    return run_affine(ctx, A, bias, h0, H, nullptr, nullptr, T, d, batch, dtype, opts, ws, ws_bytes);
}

int goom_affine_scan_scaled(goom_ctx *ctx, const void *A, const void *bias, const void *h0, void *scaled, void *logscale,
                            int64_t T, int d, int64_t batch, int dtype, const goom_scan_opts *opts, void *ws, size_t ws_bytes)
{
    if (!scaled) return fail(ctx, GOOM_EINVAL, "null data pointer");
    return run_affine(ctx, A, bias, h0, nullptr, scaled, logscale, T, d, batch, dtype, opts, ws, ws_bytes);
}

// ---- backward passes ---------------------------------------------------------------------------------------
struct AffineBackwardPlan {
    bool direct; // the adjoint scan reads the forward pass's matrices itself (transposed, in reverse order)
    bool one_matrix; // GOOM_AFFINE_TIME_INVARIANT: A is [batch, d, d] and so is its gradient
    bool same_factor; // (= one_matrix) the adjoint scan runs over A^T itself, its bias and states rescaled step by step
    int nsplit;      // one_matrix: spans of steps whose outer products are summed by one workgroup each
    size_t at_bytes, vec_bytes, scan_bytes, uv_bytes, partial_bytes;
    size_t total() const { return at_bytes + 2 * vec_bytes + scan_bytes + uv_bytes + partial_bytes; }
};

static AffineBackwardPlan plan_affine_backward(long long T, int d, long long batch, int dtype, const goom_scan_opts *opts)
{
    AffineBackwardPlan p;
    const size_t cb = 2 * comp_bytes(dtype);
    // without the time-invariant flag: the adjoint scan with shifted factors is time-varying also over one matrix
    goom_scan_opts plain = opts ? *opts : goom_scan_opts{0, 0};
    p.one_matrix = (plain.flags & GOOM_AFFINE_TIME_INVARIANT) != 0;
    plain.flags &= ~GOOM_AFFINE_TIME_INVARIANT;
    p.direct = plan_affine(T, d, batch, dtype, &plain).f64;
    p.same_factor = p.one_matrix;
    if (p.same_factor) {
        goom_scan_opts inv = plain;
        inv.flags |= GOOM_AFFINE_TIME_INVARIANT;
        p.direct = false;
        p.at_bytes = align_up((size_t)batch * d * d * cb, 256) + align_up((size_t)batch * (size_t)T * sizeof(float), 256);
        p.vec_bytes = align_up((size_t)batch * (size_t)T * d * cb, 256);
        p.scan_bytes = align_up(goom_affine_scan_workspace_bytes(T, d, batch, dtype, &inv), 256);
    } else {
        // the transposed, reversed and rescaled copy of A, or only the shifts of its log-magnitudes, one per step
        p.at_bytes = p.direct ? align_up((size_t)batch * (size_t)T * sizeof(float), 256) : align_up((size_t)batch * (size_t)T * d * d * cb, 256);
        p.vec_bytes = align_up((size_t)batch * (size_t)T * d * cb, 256);
        p.scan_bytes = align_up(goom_affine_scan_workspace_bytes(T, d, batch, dtype, &plain), 256);
    }
    p.nsplit = 1;
    p.uv_bytes = p.partial_bytes = 0;
    if (p.one_matrix) {
        // several thousand workgroups (each step's loads depend on one another: many waves in flight hide them), at least 64 steps each
        long long want = (8192 + batch - 1) / batch, most = (T + 63) / 64;
        p.nsplit = (int)(want < 1 ? 1 : want > most ? most : want);
        const int dp = d <= 16 ? 16 : d <= 32 ? 32 : d <= 64 ? 64 : 128;
        p.uv_bytes = align_up((size_t)batch * 2 * d * sizeof(double), 256); // u and v of step 0, for the initial state's gradient
        p.partial_bytes = align_up((size_t)batch * p.nsplit * dp * dp * sizeof(double), 256);
    }
    return p;
}

size_t goom_affine_scan_backward_workspace_bytes(int64_t T, int d, int64_t batch, int dtype, const goom_scan_opts *opts)
{
    if (T <= 0 || d <= 0 || batch <= 0 || d > GOOM_MAX_DIM) return 0;
    if (dtype != GOOM_C64 && dtype != GOOM_C128) return 0;
    return plan_affine_backward(T, d, batch, dtype, opts).total();
}

int goom_affine_scan_backward(goom_ctx *ctx, const void *A, const void *bias, const void *h0, const void *H, const void *grad_H,
                              void *grad_A, void *grad_bias, void *grad_h0, int64_t T, int d, int64_t batch, int dtype,
                              const goom_scan_opts *opts, void *ws, size_t ws_bytes)
{
    goom_scan_opts plain = opts ? *opts : goom_scan_opts{0, 0};
    plain.flags &= ~GOOM_AFFINE_TIME_INVARIANT; // (one matrix for all steps: A and grad_A are [batch, d, d])
    if (int s = check_scan_args(ctx, A, grad_A, T, d, 1, batch, dtype, &plain)) return s;
    if (!bias || !H || !grad_H) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (grad_h0 && !h0) return fail(ctx, GOOM_EINVAL, "a gradient for the initial state needs the initial state");
    if (d > GOOM_MAX_DIM) return fail(ctx, GOOM_EUNSUPPORTED, "the recurrence with bias needs d <= %d", GOOM_MAX_DIM);
    if (!aligned(bias, 16) || !aligned(H, 16) || (h0 && !aligned(h0, 16))) return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    const size_t rb = comp_bytes(dtype);
    if (!aligned(grad_H, rb) || !aligned(grad_A, rb) || (grad_bias && !aligned(grad_bias, rb)) || (grad_h0 && !aligned(grad_h0, rb)))
        return fail(ctx, GOOM_EINVAL, "misaligned data pointer");
    const AffineBackwardPlan p = plan_affine_backward(T, d, batch, dtype, opts);
    if (int s = check_workspace(ctx, ws, ws_bytes, p.total())) return s;
    if (int s = need_ctx(ctx)) return s;
    unsigned char *w = static_cast<unsigned char *>(ws);
    void *At = w;
    void *gt = w + p.at_bytes;
    void *mu = w + p.at_bytes + p.vec_bytes;
    void *scan_ws = w + p.at_bytes + 2 * p.vec_bytes;
    if (p.same_factor) {
        // one matrix: the adjoints lam_t themselves by the time-invariant scan over A^T, with G_t / h_t and lam_t passing through
        // the GOOM arrays on the scale e^(c_t) (the scan rescales them beside its double exponents)
        float *cshift = reinterpret_cast<float *>(w + align_up((size_t)batch * d * d * 2 * comp_bytes(dtype), 256));
        if (int s = launch_affine_backward_prepare_one_matrix(ctx, A, H, grad_H, At, cshift, gt, T, d, batch, dtype)) return s;
        goom_scan_opts inv = plain;
        inv.flags |= GOOM_AFFINE_TIME_INVARIANT;
        ctx->prof_keep = true;
        const int st = run_affine(ctx, At, gt, nullptr, mu, nullptr, nullptr, T, d, batch, dtype, &inv, p.scan_bytes ? scan_ws : nullptr, p.scan_bytes, nullptr, cshift);
        ctx->prof_keep = false;
        if (st) return st;
        unsigned char *U = w + p.at_bytes + 2 * p.vec_bytes + p.scan_bytes;
        return launch_affine_backward_gradients_one_matrix(ctx, A, bias, h0, H, mu, grad_A, grad_bias, grad_h0, U, U + p.uv_bytes, p.nsplit, T, d,
                                                           batch, dtype);
    }
    // operands of the adjoint recurrence (transposed matrices in reverse time, G / h as GOOMs) ...
    if (int s = launch_affine_backward_prepare(ctx, A, H, grad_H, p.direct ? nullptr : At, p.direct ? static_cast<float *>(At) : nullptr, gt, T, d, batch, dtype))
        return s;
    // ... the adjoints, by the forward scan itself ...
    ctx->prof_keep = true;
    const int st = p.direct ? run_affine(ctx, A, gt, nullptr, mu, nullptr, nullptr, T, d, batch, dtype, &plain, p.scan_bytes ? scan_ws : nullptr, p.scan_bytes,
                                         static_cast<const float *>(At))
                            : run_affine(ctx, At, gt, nullptr, mu, nullptr, nullptr, T, d, batch, dtype, &plain, p.scan_bytes ? scan_ws : nullptr, p.scan_bytes);
    ctx->prof_keep = false;
    if (st) return st;
    // ... and the gradients
    return launch_affine_backward_gradients(ctx, A, bias, h0, H, mu, grad_A, grad_bias, grad_h0, T, d, batch, dtype);
}

// Workspace of the LMME backward pass: the shifts, W~', both transposed operands, both products, and what the two
// forward calls ask for themselves (they run one after the other and share it).
namespace {
struct LmmeBackwardPlan {
    size_t r_bytes, c_bytes, w_bytes, at_bytes, bt_bytes, x_bytes, y_bytes, lmme_bytes;
    size_t total() const { return r_bytes + c_bytes + w_bytes + at_bytes + bt_bytes + x_bytes + y_bytes + lmme_bytes; }
};
LmmeBackwardPlan plan_lmme_backward(int64_t batch, int n, int d, int m, int dtype, uint32_t flags)
{
    const size_t rb = comp_bytes(dtype), cb = 2 * rb, bt = (size_t)batch;
    LmmeBackwardPlan p;
    p.r_bytes = align_up(bt * n * rb, 256);
    p.c_bytes = align_up(bt * m * rb, 256);
    p.w_bytes = align_up(bt * n * m * cb, 256);
    if (n == 128 && d == 128 && m == 128 && !(flags & GOOM_LMME_EXACT)) {
        // the full-size product kernel reads A and B themselves and writes the gradients: only the shifts and W~' pass through memory
        p.at_bytes = p.x_bytes = p.bt_bytes = p.y_bytes = p.lmme_bytes = 0;
        return p;
    }
    p.at_bytes = p.x_bytes = align_up(bt * n * d * cb, 256);
    p.bt_bytes = p.y_bytes = align_up(bt * d * m * cb, 256);
    const size_t wa = goom_lmme_workspace_bytes(batch, n, m, d, dtype, flags), wb = goom_lmme_workspace_bytes(batch, d, n, m, dtype, flags);
    p.lmme_bytes = align_up(wa > wb ? wa : wb, 256);
    return p;
}
} // namespace

size_t goom_lmme_backward_workspace_bytes(int64_t batch, int n, int d, int m, int dtype, uint32_t flags)
{
    if (batch <= 0 || n <= 0 || d <= 0 || m <= 0 || (dtype != GOOM_C64 && dtype != GOOM_C128)) return 0;
    if (n > GOOM_MAX_DIM_LMME || d > GOOM_MAX_DIM_LMME || m > GOOM_MAX_DIM_LMME) return 0;
    return plan_lmme_backward(batch, n, d, m, dtype, flags).total();
}

int goom_lmme_backward(goom_ctx *ctx, const void *A, const void *B, const void *Cm, const void *grad_C, void *grad_A, void *grad_B, int64_t batch, int n,
                       int d, int m, int dtype, uint32_t flags, void *ws, size_t ws_bytes)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (flags & ~GOOM_LMME_EXACT) return fail(ctx, GOOM_EINVAL, "unknown LMME flags 0x%x", flags);
    if (!A || !B || !Cm || !grad_C || !grad_A || !grad_B) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (batch <= 0 || n <= 0 || d <= 0 || m <= 0) return fail(ctx, GOOM_EINVAL, "sizes must be positive");
    if (n > GOOM_MAX_DIM_LMME || d > GOOM_MAX_DIM_LMME || m > GOOM_MAX_DIM_LMME)
        return fail(ctx, GOOM_EUNSUPPORTED, "n, d, m must be <= %d", GOOM_MAX_DIM_LMME);
    if ((lmme_is_large(n, m, d) || lmme_is_large(d, n, m)) && batch > 65535)
        return fail(ctx, GOOM_EUNSUPPORTED, "sizes above %d need batch <= 65535", GOOM_MAX_DIM);
    const int64_t widest = (int64_t)(n > d ? n : d) * (d > m ? d : m); // one workgroup per 1024 entries of a batch item, or per strip of 32 rows
    if (batch * ((widest + 1023) / 1024) > 0x7fffffffLL || batch * (((n > m ? n : m) + 31) / 32) > 0x7fffffffLL)
        return fail(ctx, GOOM_EUNSUPPORTED, "batch too large");
    if (!aligned(A, 16) || !aligned(B, 16) || !aligned(Cm, 16)) return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    const size_t rb = comp_bytes(dtype);
    if (!aligned(grad_C, rb) || !aligned(grad_A, rb) || !aligned(grad_B, rb)) return fail(ctx, GOOM_EINVAL, "misaligned data pointer");
    const LmmeBackwardPlan p = plan_lmme_backward(batch, n, d, m, dtype, flags);
    if (int s = check_workspace(ctx, ws, ws_bytes, p.total())) return s;
    if (int s = need_ctx(ctx)) return s;
    unsigned char *w = static_cast<unsigned char *>(ws);
    void *r = w;
    void *c = w + p.r_bytes;
    void *W = w + p.r_bytes + p.c_bytes;
    void *At = static_cast<unsigned char *>(W) + p.w_bytes;
    void *Bt = static_cast<unsigned char *>(At) + p.at_bytes;
    void *X = static_cast<unsigned char *>(Bt) + p.bt_bytes;
    void *Y = static_cast<unsigned char *>(X) + p.x_bytes;
    void *lw = p.lmme_bytes ? static_cast<unsigned char *>(Y) + p.y_bytes : nullptr;
    if (n == 128 && d == 128 && m == 128 && !(flags & GOOM_LMME_EXACT)) {
        // the full-size product kernel transposes and shifts its operand as it reads it and exponentiates as it stores
        if (int s = launch_lmme_backward_prepare128(ctx, A, B, Cm, grad_C, r, c, W, batch, dtype)) return s;
        if (int s = launch_lmme128_backward(ctx, 1, W, B, A, c, r, grad_A, batch, dtype)) return s;
        return launch_lmme128_backward(ctx, 2, A, W, B, r, c, grad_B, batch, dtype);
    }
    // shifts, W~' = GOOM(G) - C~', and the shifted operands transposed ...
    if (int s = launch_lmme_backward_prepare(ctx, A, B, Cm, grad_C, r, c, W, At, Bt, batch, n, d, m, dtype)) return s;
    // ... X~ = W~ B~^T [n, d] and Y~ = A~^T W~ [d, m], by the forward product itself ...
    ctx->prof_keep = true;
    int st = goom_lmme(ctx, W, Bt, X, batch, n, m, d, dtype, flags, lw, p.lmme_bytes);
    if (!st) st = goom_lmme(ctx, At, W, Y, batch, d, n, m, dtype, flags, lw, p.lmme_bytes);
    ctx->prof_keep = false;
    if (st) return st;
    // ... and the gradients A~ . X~, B~ . Y~ as reals
    return launch_lmme_backward_finish(ctx, A, B, X, Y, r, c, grad_A, grad_B, batch, n, d, m, dtype);
}

// Workspace of the scan's backward pass.  The stacked factors are dead once the reverse scan has run: the operands
// and the result of the gradient products lie in their place ((d + m)^2 >= 2 d m + d^2 entries per step).
namespace {
struct ScanBackwardPlan {
    size_t c_bytes, f_bytes, init_bytes, states_bytes, scan_bytes, lmme_bytes;
    size_t lam_off, pt_off, x_off; // inside the factors' region
    int64_t lmme_slice;            // (b, t) pairs per LMME call
    size_t total() const { return c_bytes + f_bytes + init_bytes + states_bytes + scan_bytes + lmme_bytes; }
};
ScanBackwardPlan plan_scan_backward(int64_t T, int d, int m, int64_t batch, int dtype, const goom_scan_opts *opts, bool with_init)
{
    const size_t rb = comp_bytes(dtype), cb = 2 * rb, bt = (size_t)batch;
    const int D = d + m;
    const int64_t nsteps = T + (with_init ? 1 : 0);
    ScanBackwardPlan p;
    p.c_bytes = align_up(bt * (size_t)(T + 1) * rb, 256);
    p.f_bytes = align_up(bt * (size_t)nsteps * D * D * cb, 256) + 512;
    p.init_bytes = align_up(bt * D * m * cb, 256);
    p.states_bytes = align_up(bt * (size_t)nsteps * D * m * cb, 256);
    p.scan_bytes = align_up(goom_scan_workspace_bytes(nsteps, D, m, batch, dtype, opts), 256);
    p.lam_off = 0;
    p.pt_off = align_up(bt * (size_t)T * d * m * cb, 256);
    p.x_off = p.pt_off + align_up(bt * (size_t)T * m * d * cb, 256);
    // above 128 the product takes at most 65535 pairs per call
    const bool large = d > GOOM_MAX_DIM || m > GOOM_MAX_DIM;
    p.lmme_slice = large && batch * T > 65535 ? 65535 : batch * T;
    p.lmme_bytes = align_up(goom_lmme_workspace_bytes(p.lmme_slice, d, m, d, dtype, 0), 256);
    return p;
}
} // namespace

size_t goom_scan_backward_workspace_bytes(int64_t T, int d, int m, int64_t batch, int dtype, const goom_scan_opts *opts, int with_init)
{
    if (T <= 0 || d <= 0 || m <= 0 || batch <= 0 || d + m > GOOM_MAX_DIM_LMME) return 0;
    if (dtype != GOOM_C64 && dtype != GOOM_C128) return 0;
    if (!with_init && m != d) return 0;
    return plan_scan_backward(T, d, m, batch, dtype, opts, with_init != 0).total();
}

int goom_scan_backward(goom_ctx *ctx, const void *M, const void *S0, const void *P, const void *grad_P, void *grad_M, void *grad_S0, int64_t T, int d, int m,
                       int64_t batch, int dtype, const goom_scan_opts *opts, void *ws, size_t ws_bytes)
{
    if (int s = check_scan_args(ctx, M, P, T, d, m, batch, dtype, opts, GOOM_MAX_DIM_LMME)) return s;
    if (!grad_P || !grad_M) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (!S0 && m != d) return fail(ctx, GOOM_EINVAL, "without an initial state the states are d x d (d=%d m=%d)", d, m);
    if (grad_S0 && !S0) return fail(ctx, GOOM_EINVAL, "a gradient for the initial state needs the initial state");
    if (d + m > GOOM_MAX_DIM_LMME) return fail(ctx, GOOM_EUNSUPPORTED, "the backward pass needs d + m <= %d (d=%d m=%d)", GOOM_MAX_DIM_LMME, d, m);
    if (batch * (T + 1) > 0x7fffffffLL) return fail(ctx, GOOM_EUNSUPPORTED, "batch * T too large");
    if (S0 && !aligned(S0, 16)) return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    const size_t rb = comp_bytes(dtype);
    if (!aligned(grad_P, rb) || !aligned(grad_M, rb) || (grad_S0 && !aligned(grad_S0, rb))) return fail(ctx, GOOM_EINVAL, "misaligned data pointer");
    const ScanBackwardPlan p = plan_scan_backward(T, d, m, batch, dtype, opts, S0 != nullptr);
    if (int s = check_workspace(ctx, ws, ws_bytes, p.total())) return s;
    if (int s = need_ctx(ctx)) return s;
    unsigned char *w = static_cast<unsigned char *>(ws);
    void *c = w;
    unsigned char *F = w + p.c_bytes;
    void *init = F + p.f_bytes;
    void *states = static_cast<unsigned char *>(init) + p.init_bytes;
    void *scan_ws = p.scan_bytes ? static_cast<unsigned char *>(states) + p.states_bytes : nullptr;
    void *lmme_ws = p.lmme_bytes ? static_cast<unsigned char *>(states) + p.states_bytes + p.scan_bytes : nullptr;
    const int64_t nsteps = T + (S0 ? 1 : 0);
    // scales of the states, the stacked factors [[e^(c_t - c_{t+1}) M_{t+1}^T, G_t / (P_t e^(-c_t))], [0, I]] in reverse time ...
    if (int s = launch_scan_backward_prepare(ctx, M, S0, P, grad_P, c, F, init, T, d, m, batch, dtype)) return s;
    // ... the adjoints on top of an identity, by the forward scan itself ...
    ctx->prof_keep = true;
    int st = goom_scan(ctx, F, init, states, nsteps, d + m, m, batch, dtype, opts, scan_ws, p.scan_bytes);
    // ... one product per step, adjoint times the transposed previous state ...
    void *Lam = F + p.lam_off, *Pt = F + p.pt_off, *X = F + p.x_off;
    if (!st) st = launch_scan_backward_operands(ctx, states, P, S0, c, Lam, Pt, T, d, m, batch, dtype);
    const size_t cb = 2 * rb;
    for (int64_t at = 0; !st && at < batch * T; at += p.lmme_slice) {
        const int64_t count = batch * T - at < p.lmme_slice ? batch * T - at : p.lmme_slice;
        st = goom_lmme(ctx, static_cast<unsigned char *>(Lam) + (size_t)at * d * m * cb, static_cast<unsigned char *>(Pt) + (size_t)at * m * d * cb,
                       static_cast<unsigned char *>(X) + (size_t)at * d * d * cb, count, d, m, d, dtype, GOOM_LMME_FAST, lmme_ws, p.lmme_bytes);
    }
    ctx->prof_keep = false;
    if (st) return st;
    // ... and the gradients as reals
    return launch_scan_backward_gradients(ctx, M, S0, X, states, c, grad_M, grad_S0, T, d, m, batch, dtype);
}

int goom_to_goom_backward(goom_ctx *ctx, const void *x, const void *grad_re, void *grad_x, size_t n, int dtype, double eps)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (!(eps >= 0.0)) return fail(ctx, GOOM_EINVAL, "eps must be non-negative");
    if (n == 0) return ctx ? GOOM_OK : fail(nullptr, GOOM_EINVAL, "null context");
    if (!x || !grad_re || !grad_x) return fail(ctx, GOOM_EINVAL, "null data pointer");
    const size_t al = comp_bytes(dtype);
    if (!aligned(x, al) || !aligned(grad_re, al) || !aligned(grad_x, al)) return fail(ctx, GOOM_EINVAL, "misaligned data pointer");
    if (int s = need_ctx(ctx)) return s;
    return launch_to_goom_backward(ctx, x, grad_re, grad_x, n, dtype, eps);
}

int goom_from_goom_backward(goom_ctx *ctx, const void *y, const void *grad_x, void *grad_re, size_t n, int dtype, double eps)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (!(eps >= 0.0)) return fail(ctx, GOOM_EINVAL, "eps must be non-negative");
    if (n == 0) return ctx ? GOOM_OK : fail(nullptr, GOOM_EINVAL, "null context");
    if (!y || !grad_x || !grad_re) return fail(ctx, GOOM_EINVAL, "null data pointer");
    const size_t al = comp_bytes(dtype);
    if (!aligned(y, 2 * al) || !aligned(grad_x, al) || !aligned(grad_re, al)) return fail(ctx, GOOM_EINVAL, "misaligned data pointer");
    if (int s = need_ctx(ctx)) return s;
    return launch_from_goom_backward(ctx, y, grad_x, grad_re, n, dtype, eps);
}

size_t goom_scan_reset_workspace_bytes(int64_t T, int d, int64_t batch, int dtype, const goom_reset_opts *opts)
{
    if (T <= 0 || d <= 0 || batch <= 0 || d > GOOM_MAX_DIM || (dtype != GOOM_C64 && dtype != GOOM_C128)) return 0;
    const ResetPlan p = plan_reset(T, d, batch, dtype, opts);
    return p.total();
}

int goom_scan_reset(goom_ctx *ctx, const void *J, const void *S0, void *states, uint8_t *reset_flags, double *growth,
                    int64_t T, int d, int64_t batch, int dtype, const goom_reset_opts *opts, void *workspace,
                    size_t workspace_bytes)
{
    return run_reset(ctx, J, S0, states, reset_flags, growth, 1.0, T, d, batch, dtype, opts, workspace, workspace_bytes);
}

size_t goom_scan_reset_tree_workspace_bytes(int64_t T, int d, int64_t batch, int dtype)
{
    if (T <= 0 || d <= 0 || batch <= 0 || d > GOOM_MAX_DIM || (dtype != GOOM_C64 && dtype != GOOM_C128)) return 0;
    return reset_tree_workspace_bytes(T, d, batch, dtype);
}

int goom_scan_reset_tree(goom_ctx *ctx, const void *J, const void *S0, void *states, uint8_t *reset_flags, int64_t T, int d, int64_t batch,
                         int dtype, const goom_reset_opts *opts, void *workspace, size_t workspace_bytes)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (!J || !states) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (T <= 0 || batch <= 0 || d <= 0) return fail(ctx, GOOM_EINVAL, "sizes must be positive (T=%lld d=%d batch=%lld)", (long long)T, d, (long long)batch);
    if (d > GOOM_MAX_DIM) return fail(ctx, GOOM_EUNSUPPORTED, "the reset scan supports d <= %d (d=%d)", GOOM_MAX_DIM, d);
    const int policy = opts ? opts->policy : GOOM_RESET_COLINEAR;
    if (policy < GOOM_RESET_NEVER || policy > GOOM_RESET_ALWAYS) return fail(ctx, GOOM_EINVAL, "unknown reset policy %d", policy);
    if (!aligned(J, 16) || (S0 && !aligned(S0, 16)) || !aligned(states, 16)) return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    if (int s = check_workspace(ctx, workspace, workspace_bytes, reset_tree_workspace_bytes(T, d, batch, dtype))) return s;
    if (int s = need_ctx(ctx)) return s;
    return run_reset_tree(ctx, J, S0, states, reset_flags, T, d, batch, dtype, policy, opts ? opts->cos_threshold : 0.99f, workspace);
}

int goom_lyapunov_spectrum(goom_ctx *ctx, const void *J, const void *S0, void *states, double *lambda, int64_t T, int d,
                           double dt, int64_t batch, int dtype, const goom_reset_opts *opts, void *workspace,
                           size_t workspace_bytes)
{
    if (!lambda) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (!(dt > 0.0)) return fail(ctx, GOOM_EINVAL, "dt must be positive");
    return run_reset(ctx, J, S0, states, nullptr, lambda, 1.0 / (dt * (double)T), T, d, batch, dtype, opts, workspace,
                     workspace_bytes);
}

int goom_count_nonfinite(goom_ctx *ctx, const void *z, size_t n, int dtype, uint64_t *count)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (!count || (n > 0 && !z)) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (!aligned(count, 8) || !aligned(z, 2 * comp_bytes(dtype))) return fail(ctx, GOOM_EINVAL, "misaligned data pointer");
    if (int s = need_ctx(ctx)) return s;
    return launch_count_nonfinite(ctx, z, n, dtype, reinterpret_cast<unsigned long long *>(count));
}

int goom_log_add_exp(goom_ctx *ctx, const void *x, const void *y, void *out, size_t n, int dtype)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (n == 0) return ctx ? GOOM_OK : fail(nullptr, GOOM_EINVAL, "null context");
    if (!x || !y || !out) return fail(ctx, GOOM_EINVAL, "null data pointer");
    const size_t al = 2 * comp_bytes(dtype);
    if (!aligned(x, al) || !aligned(y, al) || !aligned(out, al)) return fail(ctx, GOOM_EINVAL, "misaligned data pointer");
    if (int s = need_ctx(ctx)) return s;
    return launch_log_add_exp(ctx, x, y, out, n, dtype);
}

int goom_scaled_exp(goom_ctx *ctx, const void *z, void *scaled, void *logscale, size_t n_vectors, int d, int dtype)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (d <= 0) return fail(ctx, GOOM_EINVAL, "d must be positive");
    if (n_vectors == 0) return ctx ? GOOM_OK : fail(nullptr, GOOM_EINVAL, "null context");
    if (!z || !scaled) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (!aligned(z, 2 * comp_bytes(dtype)) || !aligned(scaled, comp_bytes(dtype)) || (logscale && !aligned(logscale, comp_bytes(dtype))))
        return fail(ctx, GOOM_EINVAL, "misaligned data pointer");
    if (int s = need_ctx(ctx)) return s;
    return launch_scaled_exp(ctx, z, scaled, logscale, n_vectors, d, dtype);
}

int goom_scaled_exp_backward(goom_ctx *ctx, const void *scaled, const void *grad_scaled, void *grad_re, size_t n, int dtype)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (n == 0) return ctx ? GOOM_OK : fail(nullptr, GOOM_EINVAL, "null context");
    if (!scaled || !grad_scaled || !grad_re) return fail(ctx, GOOM_EINVAL, "null data pointer");
    const size_t al = comp_bytes(dtype);
    if (!aligned(scaled, al) || !aligned(grad_scaled, al) || !aligned(grad_re, al)) return fail(ctx, GOOM_EINVAL, "misaligned data pointer");
    if (int s = need_ctx(ctx)) return s;
    return launch_scaled_exp_backward(ctx, scaled, grad_scaled, grad_re, n, dtype);
}

size_t goom_lyapunov_spectrum_per_step_workspace_bytes(int64_t T, int d, int64_t batch, int dtype, const goom_reset_opts *opts,
                                                       int caller_has_states, int caller_has_step_logs)
{
    if (T <= 0 || d <= 0 || batch <= 0 || d > GOOM_MAX_DIM || (dtype != GOOM_C64 && dtype != GOOM_C128)) return 0;
    const ResetPlan p = plan_reset(T, d, batch, dtype, opts);
    size_t n = p.total() + lyap_steps_partial_bytes(batch, d);
    if (!caller_has_states) n += align_up((size_t)batch * T * d * d * 2 * comp_bytes(dtype), 256);
    if (!caller_has_step_logs) n += align_up((size_t)batch * T * d * sizeof(double), 256);
    return n;
}

int goom_lyapunov_spectrum_per_step(goom_ctx *ctx, const void *J, const void *S0, void *states, double *step_logs,
                                    double *lambda, int64_t T, int d, double dt, int64_t batch, int dtype,
                                    const goom_reset_opts *opts, void *workspace, size_t workspace_bytes)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (!lambda || !J) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (!(dt > 0.0)) return fail(ctx, GOOM_EINVAL, "dt must be positive");
    if (T <= 0 || batch <= 0 || d <= 0) return fail(ctx, GOOM_EINVAL, "sizes must be positive (T=%lld d=%d batch=%lld)", (long long)T, d, (long long)batch);
    if (d > GOOM_MAX_DIM) return fail(ctx, GOOM_EUNSUPPORTED, "the reset scan supports d <= %d (d=%d)", GOOM_MAX_DIM, d);
    if (step_logs && !aligned(step_logs, 8)) return fail(ctx, GOOM_EINVAL, "step_logs must be 8-byte aligned");
    const size_t need = goom_lyapunov_spectrum_per_step_workspace_bytes(T, d, batch, dtype, opts, states != nullptr, step_logs != nullptr);
    if (int s = check_workspace(ctx, workspace, workspace_bytes, need)) return s;
    const ResetPlan p = plan_reset(T, d, batch, dtype, opts);
    unsigned char *w = static_cast<unsigned char *>(workspace) + p.total();
    double *partial = reinterpret_cast<double *>(w);
    w += lyap_steps_partial_bytes(batch, d);
    if (!states) {
        states = w;
        w += align_up((size_t)batch * T * d * d * 2 * comp_bytes(dtype), 256);
    }
    if (!step_logs) step_logs = reinterpret_cast<double *>(w);
    // group (a): all states, selectively reset
    if (int s = run_reset(ctx, J, S0, states, nullptr, nullptr, 1.0, T, d, batch, dtype, opts, workspace, p.total())) return s;
    // groups (b)-(d)
    return launch_lyap_steps(ctx, J, S0, states, step_logs, partial, lambda, T, d, batch, dtype, 1.0 / (dt * (double)T));
}

size_t goom_largest_lyapunov_workspace_bytes(int64_t T, int d, int64_t batch, int dtype, const goom_scan_opts *opts)
{
    if (T <= 0 || d <= 0 || batch <= 0 || d > GOOM_MAX_DIM) return 0;
    if (dtype != GOOM_C64 && dtype != GOOM_C128) return 0;
    const ScanPlan p = plan_scan(T, d, d, 1, batch, dtype, opts ? opts->chunk_len : 0, true);
    const size_t vec = align_up((size_t)batch * d * 2 * comp_bytes(dtype), 256);
    return align_up(p.total(), 256) + 2 * vec;
}

int goom_largest_lyapunov(goom_ctx *ctx, const void *J, const void *u0, double *lle, int64_t T, int d, double dt,
                          int64_t batch, int dtype, const goom_scan_opts *opts, void *workspace, size_t workspace_bytes)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (!lle || !J) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (!(dt > 0.0)) return fail(ctx, GOOM_EINVAL, "dt must be positive");
    if (T <= 0 || batch <= 0 || d <= 0) return fail(ctx, GOOM_EINVAL, "sizes must be positive (T=%lld d=%d batch=%lld)", (long long)T, d, (long long)batch);
    if (d > GOOM_MAX_DIM) return fail(ctx, GOOM_EUNSUPPORTED, "d must be <= %d", GOOM_MAX_DIM);
    if (!aligned(lle, 8)) return fail(ctx, GOOM_EINVAL, "lle must be 8-byte aligned");
    const size_t need = goom_largest_lyapunov_workspace_bytes(T, d, batch, dtype, opts);
    if (int s = check_workspace(ctx, workspace, workspace_bytes, need)) return s;
    const ScanPlan p = plan_scan(T, d, d, 1, batch, dtype, opts ? opts->chunk_len : 0, true);
    const size_t scan_ws = align_up(p.total(), 256);
    const size_t vec = align_up((size_t)batch * d * 2 * comp_bytes(dtype), 256);
    unsigned char *w = static_cast<unsigned char *>(workspace);
    void *final_vec = w + scan_ws;
    void *u_default = w + scan_ws + vec;
    if (!u0) {
        if (int s = need_ctx(ctx)) return s;
        if (int s = launch_uniform_u0(ctx, u_default, batch, d, dtype)) return s;
        u0 = u_default;
    }
    if (int s = run_scan(ctx, J, u0, final_vec, T, d, 1, batch, dtype, opts, workspace, scan_ws, true)) return s;
    return launch_lle_epilogue(ctx, final_vec, lle, batch, d, dtype, 1.0 / (2.0 * dt * (double)T));
}

} // extern "C"
