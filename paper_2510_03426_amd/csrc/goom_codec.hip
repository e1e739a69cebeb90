// Codec kernels: real floats <-> GOOMs (paper Section 3.1).  Pure streaming: 4 or 8
// bytes in and 8 or 16 bytes out per element (or the reverse), so HBM bandwidth binds;
// the logarithm / exponential is evaluated in double and rounded once to the component
// type, which costs nothing visible next to the memory traffic.
#include "goom_internal.h"

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

// 2 log(smallest normal): the finite stand-in for log 0 (paper Section 3.1, footnote)
constexpr double kFloorF32 = -174.67308950110621797; // 2 ln(2^-126)
constexpr double kFloorF64 = -1416.7928370645282124; // 2 ln(2^-1022)
constexpr float kPiF = 3.14159274101257324219f;
constexpr double kPiD = 3.14159265358979311600;
constexpr double kInvPi = 0.318309886183790671538;

__device__ inline float enc_re_f32(float v, bool zero_floor)
{
    if (v == 0.0f) return zero_floor ? (float)kFloorF32 : -__builtin_huge_valf();
    return (float)log((double)__builtin_fabsf(v));
}

__global__ __launch_bounds__(256) void to_goom_f32_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                          size_t n, int zero_floor)
{
    const size_t nvec = n / 4;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        f4 v = reinterpret_cast<const f4 *>(x)[i];
        f4 lo, hi;
        lo[0] = enc_re_f32(v[0], zero_floor); lo[1] = v[0] < 0.0f ? kPiF : 0.0f;
        lo[2] = enc_re_f32(v[1], zero_floor); lo[3] = v[1] < 0.0f ? kPiF : 0.0f;
        hi[0] = enc_re_f32(v[2], zero_floor); hi[1] = v[2] < 0.0f ? kPiF : 0.0f;
        hi[2] = enc_re_f32(v[3], zero_floor); hi[3] = v[3] < 0.0f ? kPiF : 0.0f;
        reinterpret_cast<f4 *>(y)[2 * i] = lo;
        reinterpret_cast<f4 *>(y)[2 * i + 1] = hi;
    }
    // ragged tail (n not a multiple of 4)
    const size_t tail0 = nvec * 4;
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid < n - tail0) {
        float v = x[tail0 + gid];
        y[2 * (tail0 + gid)] = enc_re_f32(v, zero_floor);
        y[2 * (tail0 + gid) + 1] = v < 0.0f ? kPiF : 0.0f;
    }
}

__global__ __launch_bounds__(256) void to_goom_f64_kernel(const double *__restrict__ x, double *__restrict__ y,
                                                          size_t n, int zero_floor)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        double v = x[i];
        double re = (v == 0.0) ? (zero_floor ? kFloorF64 : -__builtin_huge_val()) : log(__builtin_fabs(v));
        double2 o;
        o.x = re;
        o.y = v < 0.0 ? kPiD : 0.0;
        reinterpret_cast<double2 *>(y)[i] = o;
    }
}

__device__ inline bool odd_multiple_of_pi(double im)
{
    long long k = (long long)__builtin_rint(im * kInvPi);
    return (k & 1LL) != 0;
}

__global__ __launch_bounds__(256) void from_goom_f32_kernel(const float *__restrict__ y, float *__restrict__ x, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float2 z = reinterpret_cast<const float2 *>(y)[i];
        float mag = (float)exp((double)z.x);
        x[i] = odd_multiple_of_pi((double)z.y) ? -mag : mag;
    }
}

__global__ __launch_bounds__(256) void from_goom_f64_kernel(const double *__restrict__ y, double *__restrict__ x, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        double2 z = reinterpret_cast<const double2 *>(y)[i];
        double mag = exp(z.x);
        x[i] = odd_multiple_of_pi(z.y) ? -mag : mag;
    }
}

unsigned grid_for(size_t work_items)
{
    size_t blocks = (work_items + 255) / 256;
    const size_t cap = 256 * 32; // enough workgroups to fill 256 CUs several times over
    if (blocks > cap) blocks = cap;
    if (blocks == 0) blocks = 1;
    return (unsigned)blocks;
}

} // namespace

namespace goom {

int launch_to_goom(goom_ctx *ctx, const void *x, void *y, size_t n, int dtype, uint32_t flags)
{
    if (n == 0) return GOOM_OK;
    const int zf = (flags & GOOM_ZERO_FLOOR) ? 1 : 0;
    prof_begin(ctx, "to_goom");
    if (dtype == GOOM_C64) {
        hipLaunchKernelGGL(to_goom_f32_kernel, dim3(grid_for(n / 4 + 4)), dim3(256), 0, ctx->stream,
                           static_cast<const float *>(x), static_cast<float *>(y), n, zf);
    } else {
        hipLaunchKernelGGL(to_goom_f64_kernel, dim3(grid_for(n)), dim3(256), 0, ctx->stream,
                           static_cast<const double *>(x), static_cast<double *>(y), n, zf);
    }
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch to_goom");
}

int launch_from_goom(goom_ctx *ctx, const void *y, void *x, size_t n, int dtype)
{
    if (n == 0) return GOOM_OK;
    prof_begin(ctx, "from_goom");
    if (dtype == GOOM_C64) {
        hipLaunchKernelGGL(from_goom_f32_kernel, dim3(grid_for(n)), dim3(256), 0, ctx->stream,
                           static_cast<const float *>(y), static_cast<float *>(x), n);
    } else {
        hipLaunchKernelGGL(from_goom_f64_kernel, dim3(grid_for(n)), dim3(256), 0, ctx->stream,
                           static_cast<const double *>(y), static_cast<double *>(x), n);
    }
    prof_end(ctx);
    return check_hip(ctx, hipGetLastError(), "launch from_goom");
}

} // namespace goom
