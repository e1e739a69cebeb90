// Internal declarations shared by the libgoom sources (host side only).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>
#include <vector>

#include "../../include/goom.h"

struct goom_prof_rec {
    const char *label;
    hipEvent_t start, stop;
};

struct goom_ctx {
    int device;
    hipStream_t stream;
    std::string last_error;
    bool profile = false;
    bool prof_keep = false;               // set while one entry point runs another: timing records are not cleared
    std::vector<goom_prof_rec> prof;     // records of the last compute call
    std::vector<goom_prof_rec> prof_pool; // events kept for reuse
    void *scratch = nullptr;              // this device's copy of the library's static scratch array (goom_scan_static)
    std::string scratch_error;            // why `scratch` could not be resolved, if it could not
};

namespace goom {

int fail(goom_ctx *ctx, int status, const char *fmt, ...);
int check_hip(goom_ctx *ctx, hipError_t e, const char *what);
const char *thread_error();

// event bracketing of kernel launches (no-ops unless profiling is enabled)
void prof_reset(goom_ctx *ctx);
void prof_begin(goom_ctx *ctx, const char *label);
void prof_end(goom_ctx *ctx);

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// ---- factored matrices kept in the workspace -------------------------------------
// A running product is stored as real mantissas W[rows][cols_padded] (row-major, the
// component type of the GOOM dtype) followed by one double per padded column holding a
// power-of-two exponent: value[i][k] = W[i][k] * 2^e[k].
struct FactLayout {
    int rows_padded;   // DP: multiple of 16
    int cols_padded;   // multiple of 16
    size_t mant_bytes; // rows_padded * cols_padded * sizeof(component)
    size_t stride;     // bytes between consecutive factored matrices (256-aligned)
};
FactLayout fact_layout(int dp, int m, int dtype);
int padded_dim(int d);
// padded tile size for left factors n x d and a state of m columns: the smallest size that holds the factor
// and whose workgroup has a wave for every sixteen columns of the state
int chain_padded_dim(int n, int d, int m);

// ---- kernel launchers (defined in the .hip files) ---------------------------------
struct ChainLaunch {
    int dp;               // padded size of the tile (rows of every factored matrix); 0: chain_padded_dim(n, d, m)
    int dtype;            // GOOM_C64 / GOOM_C128
    int n;                // rows of the left factors and of the outputs (= d for chains)
    int d;                // columns of the left factors, rows of the state
    int m;                // columns of the state
    int left_fact;        // 0: left factors are GOOM matrices; 1: factored matrices (common exponent)
    int left_real;        // 1 (with left_fact = 0): left factors are real matrices of the component type
    const void *left;     // first left factor of batch item 0
    long long left_batch_stride; // bytes
    long long left_step_stride;  // bytes
    long long steps;      // left factors per batch item
    long long chunk_len;  // steps per chain (chunk); chains per batch item = ceil(steps / chunk_len)
    long long chunks_launched; // how many leading chunks per batch item get a workgroup
    long long batch;
    int init_mode;        // 0 identity, 1 factored, 2 GOOM, 3 zero
    const void *init;     // per chain (factored) or per batch item (GOOM)
    long long init_stride;       // bytes between consecutive chains (factored) / batch items (GOOM)
    long long init_group;        // > 0: factored initial states come from a grouped carry array (see goom_api.hip)
    long long init_ngroups;
    void *out_goom;       // NULL or GOOM outputs, [batch, steps, d, m]
    int out_goom_last_only;      // 1: out_goom is [batch(, chunk), d, m], written at each chain's last step
    void *out_fact_steps; // NULL or factored state before each step and after the last: (len + 1) per chain
    void *out_fact_final; // NULL or factored final state per chain
    int final_common_exponent;   // 1: out_fact_final columns share one exponent (usable as a left factor)
    long long fact_stride;       // bytes between factored matrices in out_fact_*
    int fact_cols;        // padded column count of factored states (init_mode 1, out_fact_*)
    int left_fact_cols;   // padded column count of factored left factors
    // linear recurrence with bias: one state column receives a bias vector every step
    int bias_mode;        // 0 none, 1 GOOM vectors [batch, steps, d], 2 column d of the factored left factor
    int bias_col;         // state column that receives the bias
    const void *bias;
    void *out_scaled;     // NULL or float states scaled to [-e^2, e^2], [batch, steps, d] (matrix-vector walk only)
    void *out_logscale;   // NULL or their log scales, [batch, steps]
    int io_c64;           // with dtype GOOM_C128: the GOOM arrays (left, init, bias, outputs) are complex64; the running
                          // product and every factored matrix are double
    int fact_f64;         // float kernels of the recurrence: factored matrices read / written have double mantissas
    int acc_f64;          // chunk products of the recurrence with the running product in double (float GOOM factors)
    const float *left_shift; // NULL, or [batch, steps]: factors read transposed in reverse order, log-magnitudes shifted (see ChainArgs)
    const float *io_shift;   // NULL, or [batch, steps]: bias and stored states rescaled by e^(-+io_shift[s]) (see ChainArgs)
    const char *label;    // phase name for profiling records
};
int launch_chain(goom_ctx *ctx, const ChainLaunch &a);

struct ResetLaunch {
    int dtype;            // of the GOOM arrays (s0, post_states); totals and carries always have double mantissas
    const void *totals;   // factored chunk products [batch][C]
    long long tot_stride;
    int tot_cols;
    void *carries;        // factored prefixes [batch][C + 1]
    long long car_stride;
    int car_cols;
    const void *s0;       // NULL or GOOM initial state [batch][d][d]
    void *post_states;    // NULL or GOOM states [batch][T][d][d]
    unsigned char *chunk_flags; // [batch][C] (workspace)
    unsigned char *flags; // NULL or [batch][T]
    double *growth;       // NULL or [batch][d]
    double growth_scale;
    long long T, L, C, batch;
    int d;
    int policy;
    float cos_threshold;
};
int launch_reset_carry(goom_ctx *ctx, const ResetLaunch &l);
int launch_reset_post(goom_ctx *ctx, const ResetLaunch &l);
size_t reset_tree_workspace_bytes(long long T, int d, long long batch, int dtype);
int run_reset_tree(goom_ctx *ctx, const void *J, const void *S0, void *states, unsigned char *out_flags, long long T, int d, long long batch,
                   int dtype, int policy, float cos_threshold, void *ws);
int launch_lyap_steps(goom_ctx *ctx, const void *J, const void *S0, const void *states, double *steplog, double *partial,
                      double *lambda, long long T, int d, long long batch, int dtype, double scale);
size_t lyap_steps_partial_bytes(long long batch, int d);
int launch_lle_epilogue(goom_ctx *ctx, const void *v, double *lle, long long batch, int d, int dtype, double scale);
int launch_uniform_u0(goom_ctx *ctx, void *u, long long batch, int d, int dtype);

size_t lmme_large_workspace_bytes(long long batch, int n, int d, int m);
int launch_lmme_large(goom_ctx *ctx, const void *A, const void *B, void *C, long long batch, int n, int d, int m, void *ws);
// the same for complex128 operands (double components, double-precision matrix instruction)
size_t lmme_large_f64_workspace_bytes(long long batch, int n, int d, int m);
int launch_lmme_large_f64(goom_ctx *ctx, const void *A, const void *B, void *C, long long batch, int n, int d, int m, void *ws);
// chains of matrices with 128 < d <= 256: register-resident state, one workgroup per 128 state columns
int launch_row_shifts256(goom_ctx *ctx, const void *M, float *nrow, int d, long long nmat);
int launch_chain256(goom_ctx *ctx, const void *M, const float *nrow, long long T, long long L, long long chunks, long long batch, int d, int m,
                    const float *init_s, const double *init_e, float *out_s, double *out_e, void *P);
size_t scan_large_workspace_bytes(long long T, int d, int m, long long batch, long long requested_chunk, bool final_only);
int run_scan_large(goom_ctx *ctx, const void *M, const void *init, void *P, long long T, int d, int m, long long batch,
                   long long requested_chunk, void *ws, bool final_only);
// the same for complex128 matrices
size_t scan_large_f64_workspace_bytes(long long T, int d, int m, long long batch, long long requested_chunk, bool final_only);
int run_scan_large_f64(goom_ctx *ctx, const void *M, const void *init, void *P, long long T, int d, int m, long long batch,
                       long long requested_chunk, void *ws, bool final_only);
// shifts: NULL, or [batch][2][128] in the component type: the product's final row and column shifts, written by
// launch_lmme128 and read by launch_lmme_exact (which otherwise takes the maxima of the operands itself)
int launch_lmme128(goom_ctx *ctx, const void *A, const void *B, void *C, long long batch, int dtype, void *shifts);
int launch_lmme_exact(goom_ctx *ctx, const void *A, const void *B, void *C, long long batch, int n, int d, int m, int dtype,
                      const void *shifts = nullptr);

int launch_to_goom(goom_ctx *ctx, const void *x, void *y, size_t n, int dtype, uint32_t flags);
int launch_from_goom(goom_ctx *ctx, const void *y, void *x, size_t n, int dtype);
int launch_log_add_exp(goom_ctx *ctx, const void *x, const void *y, void *out, size_t n, int dtype);
int launch_probe(goom_ctx *ctx, const void *a, void *b, size_t bytes, int mode);
int launch_matrix_probe(goom_ctx *ctx, void *sink, long long iters, int dtype);
// backward passes (goom_backward.hip)
int launch_to_goom_backward(goom_ctx *ctx, const void *x, const void *g, void *gx, size_t n, int dtype, double eps);
int launch_scaled_exp_backward(goom_ctx *ctx, const void *scaled, const void *g, void *gre, size_t n, int dtype);
int launch_from_goom_backward(goom_ctx *ctx, const void *y, const void *gx, void *g, size_t n, int dtype, double eps);
int launch_affine_backward_prepare(goom_ctx *ctx, const void *A, const void *H, const void *G, void *At, float *shift, void *gt, long long T, int d,
                                   long long batch, int dtype);
int launch_affine_backward_gradients(goom_ctx *ctx, const void *A, const void *bias, const void *h0, const void *H, const void *mu, void *gA,
                                     void *gb, void *gh0, long long T, int d, long long batch, int dtype);
// goom_lmme_tall.hip: A [batch, n, d] of many rows against B [batch, d, m] with d, m <= 64 (float components)
bool lmme_tall_applies(int n, int d, int m, int dtype);
int launch_lmme_tall(goom_ctx *ctx, const void *A, const void *B, void *Cm, long long batch, int n, int d, int m);
int launch_lmme128_backward(goom_ctx *ctx, int mode, const void *left, const void *right, const void *Z, const void *in_shift, const void *out_shift,
                            void *grad, long long batch, int dtype); // goom_lmme128.hip: a product of the backward pass with its operand transposed on the fly
// backward of LMME (goom_lmme_backward.hip): shifts r [batch, n], c [batch, m]; W [batch, n, m], At [batch, d, n], Bt [batch, m, d] GOOMs
int launch_lmme_backward_prepare(goom_ctx *ctx, const void *A, const void *B, const void *Cm, const void *G, void *r, void *c, void *W, void *At, void *Bt,
                                 long long batch, int n, int d, int m, int dtype);
int launch_lmme_backward_prepare128(goom_ctx *ctx, const void *A, const void *B, const void *Cm, const void *G, void *r, void *c, void *W, long long batch,
                                    int dtype); // n = d = m = 128: shifts and W only
int launch_lmme_backward_finish(goom_ctx *ctx, const void *A, const void *B, const void *X, const void *Y, const void *r, const void *c, void *gA, void *gB,
                                long long batch, int n, int d, int m, int dtype);
// backward of the prefix scan (goom_scan_backward.hip): c [batch, T + 1] reals; F [batch, nsteps, d + m, d + m], init [batch, d + m, m],
// states [batch, nsteps, d + m, m], Lam [batch, T, d, m], Pt [batch, T, m, d], X [batch, T, d, d] GOOMs; nsteps = T + (S0 ? 1 : 0)
int launch_scan_backward_prepare(goom_ctx *ctx, const void *M, const void *S0, const void *P, const void *G, void *c, void *F, void *init, long long T, int d,
                                 int m, long long batch, int dtype);
int launch_scan_backward_operands(goom_ctx *ctx, const void *states, const void *P, const void *S0, const void *c, void *Lam, void *Pt, long long T, int d, int m,
                                  long long batch, int dtype);
int launch_scan_backward_gradients(goom_ctx *ctx, const void *M, const void *S0, const void *X, const void *states, const void *c, void *gM, void *gS0, long long T,
                                   int d, int m, long long batch, int dtype);
int launch_affine_backward_prepare_one_matrix(goom_ctx *ctx, const void *A, const void *H, const void *G, void *At, float *shift, void *gt, long long T, int d,
                                              long long batch, int dtype); // At [batch, d, d] = A^T; shift[b, s] = c_{T-1-s}
// one matrix for all steps: gA [batch, d, d]; uv0 [batch, 2, d] doubles, partial [batch, nsplit, dp, dp] doubles (dp = d padded to 16, 32, 64, 128)
int launch_affine_backward_gradients_one_matrix(goom_ctx *ctx, const void *A, const void *bias, const void *h0, const void *H, const void *mu, void *gA,
                                                void *gb, void *gh0, void *uv0, void *partial, int nsplit, long long T, int d, long long batch, int dtype);
int launch_widen_goom(goom_ctx *ctx, const void *z64, void *z128, size_t n); // complex64 GOOMs -> complex128 GOOMs
int launch_count_nonfinite(goom_ctx *ctx, const void *z, size_t n, int dtype, unsigned long long *count);
int launch_scaled_exp(goom_ctx *ctx, const void *z, void *scaled, void *logscale, size_t nvec, int d, int dtype);

} // namespace goom

namespace goom_chain {
// time-invariant recurrence: copy A^L from the first chunk's total of every batch item to the others
int launch_replicate_power(goom_ctx *ctx, void *totals, long long stride, int fact_cols, int dp, int d, long long batch,
                           long long chunks, long long chunks_per_item, bool f64);
// recurrence with bias, float components, d = 32: every sequence walked start to end by one workgroup (goom_affine_seq.hip);
// H, scaled, logscale: any of the outputs may be NULL; adjoint_shift: NULL, or [batch, T] floats: the factor of step s is then the
// transpose of matrix T - s (any for s = 0) with adjoint_shift[s] added to its log-magnitudes
int launch_affine_seq(goom_ctx *ctx, const void *A, const void *bias, const void *h0, void *H, void *scaled, void *logscale, long long T, long long batch,
                      const float *adjoint_shift);
} // namespace goom_chain

