// C ABI of libgoom (see include/goom.h): argument validation and the host-side drivers
// that turn one call into kernel launches.  No device memory is allocated here.
#include <cmath>
#include <cstring>
#include <new>

#include "goom_internal.h"

namespace goom {

static thread_local std::string t_error;

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
    prof_reset(ctx);
    return check_hip(ctx, hipSetDevice(ctx->device), "hipSetDevice");
}

// Chunks per batch item for the three-phase scan: enough chains to fill 256 compute
// units, but not so many that the serial middle phase (one step per chunk) dominates:
// the serial depth is about 2 * chunk_len + chunks, smallest near chunks = sqrt(2 T).
static long long default_chunk_len(long long T, long long batch, long long requested)
{
    if (requested > 0) return requested < T ? requested : T;
    long long c_occ = (8192 + batch - 1) / batch;
    long long c_depth = (long long)std::ceil(std::sqrt(2.0 * (double)T));
    long long c = c_occ < c_depth ? c_occ : c_depth;
    if (c > 1024) c = 1024;
    if (c < 1) c = 1;
    long long L = (T + c - 1) / c;
    return L < 1 ? 1 : L;
}

struct ScanPlan {
    long long L, C;
    int dp;
    FactLayout tot, car;
    size_t tot_bytes, car_bytes;
};

static ScanPlan plan_scan(long long T, int d, int m_tot, int m_state, long long batch, int dtype,
                          long long requested_chunk)
{
    ScanPlan p;
    p.L = default_chunk_len(T, batch, requested_chunk);
    p.C = (T + p.L - 1) / p.L;
    p.dp = padded_dim(d);
    p.tot = fact_layout(p.dp, m_tot, dtype);
    p.car = fact_layout(p.dp, m_state, dtype);
    p.tot_bytes = p.C > 1 ? (size_t)batch * p.C * p.tot.stride : 0;
    p.car_bytes = p.C > 1 ? (size_t)batch * p.C * p.car.stride : 0;
    return p;
}

static int check_scan_args(goom_ctx *ctx, const void *M, const void *out, long long T, int d, int m, long long batch,
                           int dtype, const goom_scan_opts *opts)
{
    if (int s = check_common(ctx, dtype)) return s;
    if (!M || !out) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (T <= 0 || batch <= 0 || d <= 0 || m <= 0) return fail(ctx, GOOM_EINVAL, "sizes must be positive (T=%lld d=%d m=%d batch=%lld)", T, d, m, batch);
    if (d > GOOM_MAX_DIM || m > GOOM_MAX_DIM) return fail(ctx, GOOM_EUNSUPPORTED, "d and m must be <= %d (d=%d m=%d)", GOOM_MAX_DIM, d, m);
    if (opts && opts->flags != 0) return fail(ctx, GOOM_EINVAL, "unknown scan flags 0x%x", opts->flags);
    if (opts && opts->chunk_len < 0) return fail(ctx, GOOM_EINVAL, "negative chunk_len");
    if (!aligned(M, 16) || !aligned(out, 16)) return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    if ((d % 2) != 0 && dtype == GOOM_C64 && d != 1) { /* odd row lengths take the element-wise load path */ }
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

// scan and reduce share one driver; `final_only` selects the reduction
static int run_scan(goom_ctx *ctx, const void *M, const void *init, void *P, long long T, int d, int m, long long batch,
                    int dtype, const goom_scan_opts *opts, void *ws, size_t ws_bytes, bool final_only)
{
    if (int s = check_scan_args(ctx, M, P, T, d, m, batch, dtype, opts)) return s;
    if (!init && m != d) return fail(ctx, GOOM_EINVAL, "without an initial state the outputs are d x d (m=%d d=%d)", m, d);
    if (init && !aligned(init, 16)) return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    const ScanPlan p = plan_scan(T, d, d, m, batch, dtype, opts ? opts->chunk_len : 0);
    const size_t need = p.tot_bytes + (final_only ? 0 : p.car_bytes);
    if (int s = check_workspace(ctx, ws, ws_bytes, need)) return s;
    const size_t cb = 2 * comp_bytes(dtype);
    if (int s = need_ctx(ctx)) return s;

    ChainLaunch base;
    std::memset(&base, 0, sizeof base);
    base.dtype = dtype;
    base.n = d;
    base.d = d;
    base.batch = batch;

    if (p.C == 1) { // one chain per batch item walks everything
        ChainLaunch l = base;
        l.m = m;
        l.left = M;
        l.left_batch_stride = (long long)T * d * d * cb;
        l.left_step_stride = (long long)d * d * cb;
        l.steps = T;
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

    { // phase 1: product of every chunk (the last chunk's is needed only by the reduction)
        ChainLaunch l = base;
        l.m = d;
        l.left = M;
        l.left_batch_stride = (long long)T * d * d * cb;
        l.left_step_stride = (long long)d * d * cb;
        l.steps = T;
        l.chunk_len = p.L;
        l.chunks_launched = final_only ? p.C : p.C - 1;
        l.init_mode = 0;
        l.out_fact_final = totals;
        l.final_common_exponent = 1;
        l.fact_stride = (long long)p.tot.stride;
        l.fact_cols = p.tot.cols_padded;
        l.label = "scan_phase1_chunk_products";
        if (int s = launch_chain(ctx, l)) return s;
    }
    { // phase 2: prefixes of the chunk products (one chain per batch item)
        ChainLaunch l = base;
        l.m = m;
        l.left_fact = 1;
        l.left = totals;
        l.left_batch_stride = (long long)p.C * p.tot.stride;
        l.left_step_stride = (long long)p.tot.stride;
        l.left_fact_cols = p.tot.cols_padded;
        l.steps = final_only ? p.C : p.C - 1;
        l.chunk_len = l.steps;
        l.chunks_launched = 1;
        l.init_mode = init ? 2 : 0;
        l.init = init;
        l.init_stride = (long long)d * m * cb;
        if (final_only) {
            l.out_goom = P;
            l.out_goom_last_only = 1;
        } else {
            l.out_fact_steps = carries;
            l.fact_stride = (long long)p.car.stride;
            l.fact_cols = p.car.cols_padded;
        }
        l.label = "scan_phase2_carry_chain";
        if (int s = launch_chain(ctx, l)) return s;
        if (final_only) return GOOM_OK;
    }
    { // phase 3: every chunk again, from its incoming prefix, writing all outputs
        ChainLaunch l = base;
        l.m = m;
        l.left = M;
        l.left_batch_stride = (long long)T * d * d * cb;
        l.left_step_stride = (long long)d * d * cb;
        l.steps = T;
        l.chunk_len = p.L;
        l.chunks_launched = p.C;
        l.init_mode = 1;
        l.init = carries;
        l.init_stride = (long long)p.car.stride;
        l.fact_stride = (long long)p.car.stride;
        l.fact_cols = p.car.cols_padded;
        l.out_goom = P;
        l.label = "scan_phase3_fixup_outputs";
        return launch_chain(ctx, l);
    }
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

size_t goom_lmme_workspace_bytes(int64_t batch, int n, int d, int m, int dtype, uint32_t flags)
{
    (void)batch; (void)n; (void)d; (void)m; (void)dtype; (void)flags;
    return 0;
}

int goom_lmme(goom_ctx *ctx, const void *A, const void *B, void *C, int64_t batch, int n, int d, int m, int dtype,
              uint32_t flags, void *workspace, size_t workspace_bytes)
{
    (void)workspace; (void)workspace_bytes;
    if (int s = check_common(ctx, dtype)) return s;
    if (flags & ~GOOM_LMME_EXACT) return fail(ctx, GOOM_EINVAL, "unknown LMME flags 0x%x", flags);
    if (!A || !B || !C) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (batch <= 0 || n <= 0 || d <= 0 || m <= 0) return fail(ctx, GOOM_EINVAL, "sizes must be positive");
    if (n > GOOM_MAX_DIM || d > GOOM_MAX_DIM || m > GOOM_MAX_DIM) return fail(ctx, GOOM_EUNSUPPORTED, "n, d, m must be <= %d", GOOM_MAX_DIM);
    if (!aligned(A, 16) || !aligned(B, 16) || !aligned(C, 16)) return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    if (flags & GOOM_LMME_EXACT) return fail(ctx, GOOM_EUNSUPPORTED, "GOOM_LMME_EXACT is not built yet");
    if (int s = need_ctx(ctx)) return s;
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
    return launch_chain(ctx, l);
}

size_t goom_scan_workspace_bytes(int64_t T, int d, int m, int64_t batch, int dtype, const goom_scan_opts *opts)
{
    if (T <= 0 || d <= 0 || m <= 0 || batch <= 0 || d > GOOM_MAX_DIM || m > GOOM_MAX_DIM) return 0;
    if (dtype != GOOM_C64 && dtype != GOOM_C128) return 0;
    ScanPlan p = plan_scan(T, d, d, m, batch, dtype, opts ? opts->chunk_len : 0);
    return p.tot_bytes + p.car_bytes;
}

size_t goom_reduce_workspace_bytes(int64_t T, int d, int m, int64_t batch, int dtype, const goom_scan_opts *opts)
{
    if (T <= 0 || d <= 0 || m <= 0 || batch <= 0 || d > GOOM_MAX_DIM || m > GOOM_MAX_DIM) return 0;
    if (dtype != GOOM_C64 && dtype != GOOM_C128) return 0;
    ScanPlan p = plan_scan(T, d, d, m, batch, dtype, opts ? opts->chunk_len : 0);
    return p.tot_bytes;
}

int goom_scan(goom_ctx *ctx, const void *M, const void *init, void *P, int64_t T, int d, int m, int64_t batch, int dtype,
              const goom_scan_opts *opts, void *workspace, size_t workspace_bytes)
{
    return run_scan(ctx, M, init, P, T, d, m, batch, dtype, opts, workspace, workspace_bytes, false);
}

int goom_reduce(goom_ctx *ctx, const void *M, const void *init, void *P_final, int64_t T, int d, int m, int64_t batch,
                int dtype, const goom_scan_opts *opts, void *workspace, size_t workspace_bytes)
{
    return run_scan(ctx, M, init, P_final, T, d, m, batch, dtype, opts, workspace, workspace_bytes, true);
}

size_t goom_affine_scan_workspace_bytes(int64_t T, int d, int64_t batch, int dtype, const goom_scan_opts *opts)
{
    if (T <= 0 || d <= 0 || batch <= 0 || d >= GOOM_MAX_DIM) return 0;
    if (dtype != GOOM_C64 && dtype != GOOM_C128) return 0;
    ScanPlan p = plan_scan(T, d, d + 1, 1, batch, dtype, opts ? opts->chunk_len : 0);
    return p.tot_bytes + p.car_bytes;
}

int goom_affine_scan(goom_ctx *ctx, const void *A, const void *bias, const void *h0, void *H, int64_t T, int d,
                     int64_t batch, int dtype, const goom_scan_opts *opts, void *ws, size_t ws_bytes)
{
    if (int s = check_scan_args(ctx, A, H, T, d, 1, batch, dtype, opts)) return s;
    if (!bias) return fail(ctx, GOOM_EINVAL, "null data pointer");
    if (d >= GOOM_MAX_DIM) return fail(ctx, GOOM_EUNSUPPORTED, "the recurrence with bias needs d < %d", GOOM_MAX_DIM);
    if (!aligned(bias, 16) || (h0 && !aligned(h0, 16))) return fail(ctx, GOOM_EINVAL, "complex data must be 16-byte aligned");
    const ScanPlan p = plan_scan(T, d, d + 1, 1, batch, dtype, opts ? opts->chunk_len : 0);
    if (int s = check_workspace(ctx, ws, ws_bytes, p.tot_bytes + p.car_bytes)) return s;
    if (int s = need_ctx(ctx)) return s;
    const size_t cb = 2 * comp_bytes(dtype);

    ChainLaunch base;
    std::memset(&base, 0, sizeof base);
    base.dtype = dtype;
    base.n = d;
    base.d = d;
    base.batch = batch;
    base.left = A;
    base.left_batch_stride = (long long)T * d * d * cb;
    base.left_step_stride = (long long)d * d * cb;
    base.steps = T;
    base.bias_mode = 1;
    base.bias = bias;

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
    { // phase 1: augmented chunk products [A* | b*]
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
        l.label = "affine_phase1_chunk_products";
        if (int s = launch_chain(ctx, l)) return s;
    }
    { // phase 2: h at the chunk boundaries
        ChainLaunch l;
        std::memset(&l, 0, sizeof l);
        l.dtype = dtype;
        l.n = d;
        l.d = d;
        l.m = 1;
        l.batch = batch;
        l.left_fact = 1;
        l.left = totals;
        l.left_batch_stride = (long long)p.C * p.tot.stride;
        l.left_step_stride = (long long)p.tot.stride;
        l.left_fact_cols = p.tot.cols_padded;
        l.steps = p.C - 1;
        l.chunk_len = p.C - 1;
        l.chunks_launched = 1;
        l.init_mode = h0 ? 2 : 3;
        l.init = h0;
        l.init_stride = (long long)d * cb;
        l.bias_mode = 2;
        l.bias_col = 0;
        l.out_fact_steps = carries;
        l.fact_stride = (long long)p.car.stride;
        l.fact_cols = p.car.cols_padded;
        l.label = "affine_phase2_carry_chain";
        if (int s = launch_chain(ctx, l)) return s;
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
        l.fact_stride = (long long)p.car.stride;
        l.fact_cols = p.car.cols_padded;
        l.out_goom = H;
        l.label = "affine_phase3_outputs";
        return launch_chain(ctx, l);
    }
}

size_t goom_scan_reset_workspace_bytes(int64_t T, int d, int64_t batch, int dtype, const goom_reset_opts *opts)
{
    (void)T; (void)d; (void)batch; (void)dtype; (void)opts;
    return 0;
}

int goom_scan_reset(goom_ctx *ctx, const void *J, const void *S0, void *states, uint8_t *reset_flags, double *growth,
                    int64_t T, int d, int64_t batch, int dtype, const goom_reset_opts *opts, void *workspace,
                    size_t workspace_bytes)
{
    (void)J; (void)S0; (void)states; (void)reset_flags; (void)growth; (void)T; (void)d; (void)batch; (void)opts;
    (void)workspace; (void)workspace_bytes;
    if (int s = check_common(ctx, dtype)) return s;
    return fail(ctx, GOOM_EUNSUPPORTED, "goom_scan_reset is not built yet");
}

int goom_lyapunov_spectrum(goom_ctx *ctx, const void *J, const void *S0, void *states, double *lambda, int64_t T, int d,
                           double dt, int64_t batch, int dtype, const goom_reset_opts *opts, void *workspace,
                           size_t workspace_bytes)
{
    (void)J; (void)S0; (void)states; (void)lambda; (void)T; (void)d; (void)dt; (void)batch; (void)opts;
    (void)workspace; (void)workspace_bytes;
    if (int s = check_common(ctx, dtype)) return s;
    return fail(ctx, GOOM_EUNSUPPORTED, "goom_lyapunov_spectrum is not built yet");
}

} // extern "C"
