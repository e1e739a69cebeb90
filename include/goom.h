/*
 * goom.h -- C ABI of libgoom: parallel prefix scans over chains of real matrices held
 * as generalized orders of magnitude (GOOMs), for one AMD MI355X (gfx950).
 *
 * A GOOM is a complex logarithm x' of a real number x = exp(x'): the real part is
 * log|x|, the imaginary part is 0 for x >= 0 and pi for x < 0 (paper Section 2; zero
 * is the non-negative GOOM with real part -inf).  Arrays of GOOMs use the interleaved
 * complex layout (re, im): GOOM_C64 has float components, GOOM_C128 double components
 * (paper Section 3).
 *
 * Conventions for every call
 *   - C linkage, plain pointers and sizes; no exception crosses the boundary.
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library reads
 *     inputs, writes outputs and the caller-provided workspace, and keeps none of them
 *     after the enqueued work has finished.  It never allocates or frees device memory.
 *   - Work is enqueued on the context's HIP stream and is asynchronous: results are
 *     valid once the caller has synchronised that stream.  Inputs are never modified;
 *     outputs and the workspace may not overlap inputs or each other.
 *   - Matrices are row-major with the innermost index contiguous; a leading "batch"
 *     index runs over independent problems (paper Section 3: functions broadcast over
 *     preceding indices).  Complex data must be 16-byte aligned, real data aligned to
 *     its element size, the workspace to 256 bytes.
 *   - Return value: GOOM_OK or a negative goom_status.  goom_last_error(ctx) returns a
 *     message for the last failure on that context (thread-local when ctx is NULL).
 *     Arguments are validated on the host before anything is enqueued; a failed call
 *     enqueues nothing.
 *   - Only imaginary parts 0 and pi (of the component type) are ever written.  On input
 *     any multiple of pi is accepted; the sign is the parity of round(im / pi).
 *   - Non-finite log-magnitudes other than -inf (that is +inf and NaN) are outside the
 *     contract of the product calls.
 *
 * Range of the product calls.  Inside a product the factors are exponentiated after a
 * per-row shift of the left factor and a per-column shift of the right factor (paper
 * Section 3.2, eq. 10), so within one row-by-column sum terms smaller than the largest
 * possible term by more than the component format's range (about e^-87 for GOOM_C64,
 * e^-708 for GOOM_C128) are dropped, as in the paper's own implementation.
 * goom_lmme can be asked to repair such sums exactly (GOOM_LMME_EXACT).
 */
#ifndef GOOM_H
#define GOOM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
#pragma GCC visibility push(default)

#define GOOM_VERSION 100 /* major * 10000 + minor * 100 + patch */

typedef struct goom_ctx goom_ctx;

typedef enum goom_status {
    GOOM_OK = 0,
    GOOM_EINVAL = -1,       /* null pointer, non-positive size, bad flag, misalignment */
    GOOM_EUNSUPPORTED = -2, /* valid request outside what this build implements */
    GOOM_EWORKSPACE = -3,   /* workspace missing or smaller than *_workspace_bytes */
    GOOM_EHIP = -4,         /* a HIP runtime call failed (message has the HIP error) */
    GOOM_ENOMEM = -5        /* host allocation failed */
} goom_status;

typedef enum goom_dtype {
    GOOM_C64 = 0, /* complex64: float log-magnitude, float phase */
    GOOM_C128 = 1 /* complex128: double log-magnitude, double phase */
} goom_dtype;

/* largest matrix dimension of the register-resident kernels (scans, recurrences, small products) */
#define GOOM_MAX_DIM 128
/* largest dimension of goom_lmme, goom_scan and goom_reduce (both formats): above GOOM_MAX_DIM the
 * product runs as scaled operands, a tiled GEMM and a store pass through the workspace (the paper's experiments
 * go up to 1024) */
#define GOOM_MAX_DIM_LMME 1024

/* flags of goom_to_goom: how log 0 is written (paper Section 3.1, configurable real log) */
#define GOOM_ZERO_NEG_INF 0u /* log 0 = -inf (default) */
#define GOOM_ZERO_FLOOR 1u   /* log 0 = 2 log(smallest normal): finite, exponentiates to 0 */

/* flags of goom_lmme */
#define GOOM_LMME_FAST 0u  /* scaled real product only (paper Section 3.2, eq. 10) */
#define GOOM_LMME_EXACT 1u /* additionally recompute, by a signed log-sum-exp over the
                              terms (eq. 9, the definition), every output whose scaled product lost
                              terms to underflow */

/* ---- context ------------------------------------------------------------------- */

int goom_version(void);

/* Create a context bound to HIP device `device` and to `stream` (a hipStream_t passed as
 * void*; NULL = the device's default stream).  The stream stays owned by the caller.
 * Fails with GOOM_EHIP when the device cannot be used. */
int goom_create(goom_ctx **ctx, int device, void *stream);
int goom_destroy(goom_ctx *ctx);
int goom_set_stream(goom_ctx *ctx, void *stream);
const char *goom_last_error(const goom_ctx *ctx);
const char *goom_status_name(int status);

/* ---- per-kernel timing (measurement aid, not part of the method) ------------------- */

/* When enabled, every kernel a compute call enqueues is bracketed by HIP events on the
 * context's stream.  Records are cleared at the start of each compute call.
 * goom_profile_get waits for record i of the last call and returns the kernel's label
 * (a static string naming the phase) and its elapsed time in milliseconds. */
int goom_profile_enable(goom_ctx *ctx, int enable);
int goom_profile_count(const goom_ctx *ctx);
int goom_profile_get(goom_ctx *ctx, int i, const char **label, float *milliseconds);

/* What this device's memory system sustains for plain streaming, for setting a kernel's achieved
 * rate beside something measured (measurement aid, not part of the method).  Enqueues one
 * pass over `bytes` bytes (a multiple of 16; a, b 16-byte aligned device buffers of that size):
 * GOOM_PROBE_READ reads a (b receives 4 bytes), GOOM_PROBE_WRITE fills b, GOOM_PROBE_COPY copies
 * a to b.  The caller times it on the context's stream. */
#define GOOM_PROBE_READ 0
#define GOOM_PROBE_WRITE 1
#define GOOM_PROBE_COPY 2
int goom_probe_bandwidth(goom_ctx *ctx, const void *a, void *b, size_t bytes, int mode);

/* What the matrix units sustain when a kernel issues nothing else (measurement aid): enqueues a kernel of
 * 2048 workgroups x 4 waves, each wave issuing 8 x `iters` 16 x 16 x 4 matrix instructions (2048 flop each)
 * in the component type of `dtype` (float for GOOM_C64, double for GOOM_C128) on independent accumulators:
 * GOOM_PROBE_MATRIX_FLOP_PER_ITER x iters flop in all.  sink: at least 4 bytes of device memory (never
 * written in practice).  The caller times it on the context's stream. */
#define GOOM_PROBE_MATRIX_FLOP_PER_ITER 134217728LL /* 2048 workgroups x 4 waves x 8 instructions x 2048 flop */
int goom_probe_matrix_unit(goom_ctx *ctx, void *sink, int64_t iters, int dtype);

/* ---- codecs (paper Section 3.1) -------------------------------------------------- */

/* Real floats -> GOOMs: y[i] = (log|x[i]|, x[i] < 0 ? pi : 0).  x: n floats (GOOM_C64)
 * or n doubles (GOOM_C128); y: n complex.  The logarithm is rounded once from a
 * higher-precision evaluation.  +-0 -> (-inf, 0) or (floor, 0) per `flags`;
 * NaN -> (NaN, 0); +-inf -> (+inf, 0 or pi).  n = 0 is a no-op. */
int goom_to_goom(goom_ctx *ctx, const void *x, void *y, size_t n, int dtype, uint32_t flags);

/* GOOMs -> real floats: x[i] = +-exp(Re y[i]), the real part of the complex exponential
 * (paper Section 3.1, eq. 7); overflow gives +-inf, underflow +-0. */
int goom_from_goom(goom_ctx *ctx, const void *y, void *x, size_t n, int dtype);

/* Number of entries of a GOOM array whose log-magnitude is +inf or NaN (-inf, the GOOM of zero, is finite): the
 * paper's notion of a failed chain is one that ends in non-finite values (Section 4.1).  z: n GOOMs; count: one
 * device uint64, overwritten.  Reads z once; an optional check after any of the product calls. */
int goom_count_nonfinite(goom_ctx *ctx, const void *z, size_t n, int dtype, uint64_t *count);

/* ---- LMME (paper Section 3.2) ---------------------------------------------------- */

/* C[b] = LMME(A[b], B[b]) = log(exp(A[b]) exp(B[b])) for b < batch.
 * A: [batch, n, d], B: [batch, d, m], C: [batch, n, m] GOOMs; 1 <= n, d, m <= GOOM_MAX_DIM_LMME
 * (above GOOM_MAX_DIM the workspace is required, and batch <= 65535).
 * Computed as the paper's scaled real product on the matrix cores (eq. 10) with row
 * shifts max_j Re A_ij and column shifts max_j Re B_jk (0 for an all-zero row/column).
 * A sum that is exactly zero gives (-inf, 0).  flags: GOOM_LMME_FAST or GOOM_LMME_EXACT.
 * workspace: goom_lmme_workspace_bytes(...) bytes (may be 0 -> NULL allowed).  For n = d = m = 128 with
 * GOOM_LMME_EXACT the query asks for 256 components per pair, in which the product hands its row and
 * column shifts to the repair pass; there the workspace is optional (NULL or a smaller one: the repair
 * pass takes the maxima of the operands itself, more slowly, with the same results within tolerance). */
int goom_lmme(goom_ctx *ctx, const void *A, const void *B, void *C, int64_t batch, int n, int d,
              int m, int dtype, uint32_t flags, void *workspace, size_t workspace_bytes);
size_t goom_lmme_workspace_bytes(int64_t batch, int n, int d, int m, int dtype, uint32_t flags);

/* ---- prefix scan of a chain of matrix products (paper Section 4.1; Section 4.2.2) -- */

typedef struct goom_scan_opts {
    int64_t chunk_len; /* matrices per chunk of the three-phase scan; 0 = library default */
    uint32_t flags;    /* 0, or GOOM_AFFINE_TIME_INVARIANT for goom_affine_scan */
} goom_scan_opts;

/* Inclusive prefix products, newer factor on the left (paper Section 4.1, eq. 14):
 *     P[b, 0] = LMME(M[b, 0], init[b])      (or M[b, 0] itself when init is NULL)
 *     P[b, t] = LMME(M[b, t], P[b, t-1])
 * M: [batch, T, d, d]; init: NULL or [batch, d, m] (m != d allowed, e.g. a vector u_0,
 * m = 1); P: [batch, T, d, m] (m = d when init is NULL); 1 <= d, m <= GOOM_MAX_DIM_LMME, both
 * formats.  opts may be NULL.
 * The chain is cut into chunks: phase 1 multiplies each chunk down to one matrix,
 * phase 2 scans those chunk products, phase 3 re-walks every chunk from its incoming
 * prefix and writes all outputs.  Between steps the running product is kept as real
 * mantissas with a power-of-two exponent per column, so log-magnitudes are rounded to
 * the component type only when an output is stored.
 * workspace: goom_scan_workspace_bytes(...) bytes. */
int goom_scan(goom_ctx *ctx, const void *M, const void *init, void *P, int64_t T, int d, int m,
              int64_t batch, int dtype, const goom_scan_opts *opts, void *workspace,
              size_t workspace_bytes);
size_t goom_scan_workspace_bytes(int64_t T, int d, int m, int64_t batch, int dtype,
                                 const goom_scan_opts *opts);

/* goom_scan for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the scan's workspace is a static array of
 * GOOM_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until the process ends; the call
 * itself allocates nothing.  Arguments and results as for goom_scan (same kernels, same launch plan,
 * bit-identical outputs).  If the default plan (opts NULL or chunk_len 0) needs more than the array holds,
 * the shortest chunk length among 8, 16, 32, ... whose plan fits is taken instead (the outputs are then those of
 * goom_scan with that chunk_len).  A scan whose goom_scan_workspace_bytes(...) still exceeds
 * GOOM_STATIC_SCRATCH_BYTES is rejected with GOOM_EWORKSPACE and nothing is enqueued (the T = 2^20, d = 64
 * complex64 scan needs 36.2 MB and fits).  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two contexts, two threads) race on it and must be serialised by the caller.  Nothing in the array
 * has to be cleared between calls: every phase writes what the next one reads. */
#define GOOM_STATIC_SCRATCH_BYTES (40u << 20)
int goom_scan_static(goom_ctx *ctx, const void *M, const void *init, void *P, int64_t T, int d, int m,
                     int64_t batch, int dtype, const goom_scan_opts *opts);

/* Only the last prefix: P_final[b] = P[b, T-1] of goom_scan ([batch, d, m]); phases 1 and
 * 2 only, so the input is read once (the product inside the paper's largest-exponent
 * formula, Section 4.2.2, eq. 24). */
int goom_reduce(goom_ctx *ctx, const void *M, const void *init, void *P_final, int64_t T, int d,
                int m, int64_t batch, int dtype, const goom_scan_opts *opts, void *workspace,
                size_t workspace_bytes);
size_t goom_reduce_workspace_bytes(int64_t T, int d, int m, int64_t batch, int dtype,
                                   const goom_scan_opts *opts);

/* The same scan and reduction over REAL matrices X: [batch, T, d, d] of the component type (floats for
 * GOOM_C64), i.e. goom_scan(goom_to_goom(X)) without the encoded copy of the input: chains usually start
 * from real matrices (paper Section 4.1 draws them from N(0, 1)), and reading them directly halves the
 * input traffic.  For GOOM_C64 with d = 32, 64 or 128 and a square state the chain kernel reads the reals
 * itself and scales an entry by its powers of two exactly (no logarithm or exponential on the way in, so
 * the result is that of the scan over exactly encoded inputs); other shapes are encoded into the
 * workspace first.  init, P, opts as for goom_scan.  workspace: goom_scan_real_workspace_bytes(...) /
 * goom_reduce_real_workspace_bytes(...) bytes. */
int goom_scan_real(goom_ctx *ctx, const void *X, const void *init, void *P, int64_t T, int d, int m,
                   int64_t batch, int dtype, const goom_scan_opts *opts, void *workspace,
                   size_t workspace_bytes);
size_t goom_scan_real_workspace_bytes(int64_t T, int d, int m, int64_t batch, int dtype,
                                      const goom_scan_opts *opts);
int goom_reduce_real(goom_ctx *ctx, const void *X, const void *init, void *P_final, int64_t T, int d,
                     int m, int64_t batch, int dtype, const goom_scan_opts *opts, void *workspace,
                     size_t workspace_bytes);
size_t goom_reduce_real_workspace_bytes(int64_t T, int d, int m, int64_t batch, int dtype,
                                        const goom_scan_opts *opts);

/* ---- selectively reset scan and Lyapunov spectrum (paper Section 5; Section 4.2.1) - */

#define GOOM_RESET_ALWAYS 1     /* reset at every examined state */
#define GOOM_RESET_COLINEAR 0   /* reset when any two columns have |cosine| > threshold */
#define GOOM_RESET_NEVER (-1)   /* plain scan */

typedef struct goom_reset_opts {
    int64_t chunk_len;    /* states are examined every chunk_len steps (t = chunk_len,
                             2 chunk_len, ...); 0 = library default (128).  Longer chunks shorten
                             the serial phase; between two examined states the columns may close
                             in on each other by a factor of about 1e5 (the spread of the
                             exponents times chunk_len dt, as a power of e) before the
                             factorisation, which runs in double, loses accuracy */
    int32_t policy;       /* GOOM_RESET_* */
    float cos_threshold;  /* used by GOOM_RESET_COLINEAR */
} goom_reset_opts;

/* X[b, t] = J[b, t] X[b, t-1], t = 0..T-1 in array terms, X[b, -1] = S0[b] (NULL =
 * identity), over GOOMs, with the selective-resetting method applied to the true
 * prefix states at chunk boundaries: a selected state is replaced by the orthonormal
 * factor Q of its column-normalised real form (paper Section 4.2.1 (a)), and all later
 * states continue from Q.
 * Both formats, d <= 128 (goom_lyapunov_spectrum as well).  Chunk products, the prefixes at the chunk boundaries and the
 * factorisations are computed in double for both formats; complex64 states are rounded once,
 * when they are stored.
 * J: [batch, T, d, d]; S0: NULL or [batch, d, d]; states: [batch, T, d, d] (the state
 * after any reset at that step); reset_flags: NULL or [batch, T] bytes (1 where a reset
 * happened); growth: NULL or [batch, d] doubles: per column, the sum over resets of
 * log R_kk + log(column norm), plus the same for the final state, i.e. the total
 * log-growth of the k-th orthogonalised direction.
 * workspace: goom_scan_reset_workspace_bytes(...) bytes. */
int goom_scan_reset(goom_ctx *ctx, const void *J, const void *S0, void *states,
                    uint8_t *reset_flags, double *growth, int64_t T, int d, int64_t batch,
                    int dtype, const goom_reset_opts *opts, void *workspace,
                    size_t workspace_bytes);
size_t goom_scan_reset_workspace_bytes(int64_t T, int d, int64_t batch, int dtype,
                                       const goom_reset_opts *opts);

/* The same recurrence with the selective-resetting transformation applied in the order of the paper's own
 * parallel prefix scan (Section 5, eq. 28; Appendix C): elements (X_0, J_0, ..., J_{T-1}); parallel step k updates
 * the upper half of every block of 2^k elements from the last element of its lower half; before every parallel
 * step each interim compound that S selects (opts->policy, opts->cos_threshold; chunk_len is not used) and that
 * has not been reset yet is replaced by R of itself and from then on ignores what precedes it.  Which compounds
 * exist depends on this order, so the result differs from goom_scan_reset's (both are instances of the paper's
 * method); a compound that does not contain X_0 carries no history, and resetting it discards the earlier
 * states' subspaces, which is why goom_scan_reset, not this call, serves the spectrum estimators.  O(T log T)
 * products.  states: [batch, T, d, d] (the paper's "Sums"); reset_flags: NULL or [batch, T] bytes, 1 where the
 * final value of a state descends from a reset.  Both formats, d <= 128.
 * workspace: goom_scan_reset_tree_workspace_bytes(...) bytes. */
int goom_scan_reset_tree(goom_ctx *ctx, const void *J, const void *S0, void *states, uint8_t *reset_flags,
                         int64_t T, int d, int64_t batch, int dtype, const goom_reset_opts *opts, void *workspace,
                         size_t workspace_bytes);
size_t goom_scan_reset_tree_workspace_bytes(int64_t T, int d, int64_t batch, int dtype);

/* Lyapunov spectrum from the reset scan: lambda[b, k] = growth[b, k] / (dt T)
 * (paper Section 4.2.1, eq. 20, with the triangular factors accumulated at the resets).  states is
 * optional here (NULL = do not store them).  lambda: [batch, d] doubles. */
int goom_lyapunov_spectrum(goom_ctx *ctx, const void *J, const void *S0, void *states,
                           double *lambda, int64_t T, int d, double dt, int64_t batch, int dtype,
                           const goom_reset_opts *opts, void *workspace, size_t workspace_bytes);

/* Lyapunov spectrum by the paper's four groups of parallel computations (Section 4.2.1
 * (a)-(d)): (a) the selectively reset scan above gives the input states S_0 .. S_{T-1};
 * (b) each is log-scaled and factorised, S_{t-1} -> Q_{t-1}; (c) S*_t = J_t Q_{t-1};
 * (d) S*_t -> R_t, and lambda[b, k] = mean over t of log R_t,kk / dt.  Every step of (b)-(d)
 * is independent of the others.  states: NULL or [batch, T, d, d] (as in goom_scan_reset);
 * step_logs: NULL or [batch, T, d] doubles receiving log R_t,kk; lambda: [batch, d] doubles.
 * Both formats (complex128, and both formats above d = 64: factorisations and products in double), d <= 128.
 * workspace: goom_lyapunov_spectrum_per_step_workspace_bytes(..., states != NULL,
 * step_logs != NULL) bytes. */
int goom_lyapunov_spectrum_per_step(goom_ctx *ctx, const void *J, const void *S0, void *states,
                                    double *step_logs, double *lambda, int64_t T, int d, double dt,
                                    int64_t batch, int dtype, const goom_reset_opts *opts,
                                    void *workspace, size_t workspace_bytes);
size_t goom_lyapunov_spectrum_per_step_workspace_bytes(int64_t T, int d, int64_t batch, int dtype,
                                                       const goom_reset_opts *opts,
                                                       int caller_has_states, int caller_has_step_logs);

/* Largest Lyapunov exponent (paper Section 4.2.2): lle[b] = LSE(2 v') / (2 dt T) with
 * v' the GOOM vector J[b, T-1] ... J[b, 0] u0[b], computed as a reduction over the chain.
 * J: [batch, T, d, d]; u0: NULL (all entries 1 / sqrt(d)) or [batch, d] GOOMs; lle: [batch]
 * doubles.  workspace: goom_largest_lyapunov_workspace_bytes(...) bytes. */
int goom_largest_lyapunov(goom_ctx *ctx, const void *J, const void *u0, double *lle, int64_t T,
                          int d, double dt, int64_t batch, int dtype, const goom_scan_opts *opts,
                          void *workspace, size_t workspace_bytes);
size_t goom_largest_lyapunov_workspace_bytes(int64_t T, int d, int64_t batch, int dtype,
                                             const goom_scan_opts *opts);

/* ---- linear recurrence with bias (paper Section 4.3, eqs. 25 and 26) ---------------- */

/* Signed log-add, elementwise: out[i] is the GOOM of exp(x[i]) + exp(y[i]) (paper Section 2,
 * Example 2; the step that adds the input term in eq. 26).  x, y, out: n GOOMs each; out may
 * alias x or y.  Equal magnitudes of opposite sign give zero, (-inf, 0). */
int goom_log_add_exp(goom_ctx *ctx, const void *x, const void *y, void *out, size_t n, int dtype);

/* Scaled exponentiation of GOOM vectors (paper Section 4.3, eq. 27), the way recurrence states
 * return to a floating-point format: for each of n_vectors vectors z[v, 0..d-1],
 * c = max_i Re z[v, i] and scaled[v, i] = (+-) exp(Re z[v, i] - c + 2), so all results lie in
 * [-e^2, e^2] whatever the magnitude of the state.  z: [n_vectors, d] GOOMs; scaled:
 * [n_vectors, d] reals of the component type; logscale: NULL or [n_vectors] reals receiving c
 * (-inf for a vector of zeros, whose scaled entries are 0). */
int goom_scaled_exp(goom_ctx *ctx, const void *z, void *scaled, void *logscale, size_t n_vectors,
                    int d, int dtype);


/* h[b, t] = A[b, t] h[b, t-1] + bias[b, t], h[b, -1] = h0[b] (NULL = zero vector), over
 * GOOMs.  A: [batch, T, d, d]; bias: [batch, T, d]; h0: NULL or [batch, d];
 * H: [batch, T, d].  Scanned as products of the augmented matrices [A | bias; 0 | 1]
 * whose last row is kept implicit.  A batch of 96 sequences or more with a matrix per step,
 * float components, d = 32 and opts->chunk_len == 0 is not scanned: every sequence is walked
 * start to end by one workgroup, every matrix read once (the results are those of a sequential
 * float evaluation; whole-number exponents are kept within +-2^28, i.e. log-magnitudes within
 * +-1.8e8, beyond which a float log-magnitude resolves nothing anyway).
 * workspace: goom_affine_scan_workspace_bytes(...) bytes. */
#define GOOM_AFFINE_TIME_INVARIANT 0x1u /* goom_scan_opts.flags: one matrix per batch item, A: [batch, d, d],
                                           applied at every step (the paper's state-space layer has constant
                                           A); it is encoded once and its powers serve all chunks */
int goom_affine_scan(goom_ctx *ctx, const void *A, const void *bias, const void *h0, void *H,
                     int64_t T, int d, int64_t batch, int dtype, const goom_scan_opts *opts,
                     void *workspace, size_t workspace_bytes);
size_t goom_affine_scan_workspace_bytes(int64_t T, int d, int64_t batch, int dtype,
                                        const goom_scan_opts *opts);

/* The same recurrence with its states returned in scaled floating-point form (paper Section 4.3,
 * eq. 27), the format the layers after the recurrence consume: scaled[b, t, i] =
 * (+-) exp(Re h[b, t, i] - c[b, t] + 2) with c[b, t] = max_i Re h[b, t, i], all within
 * [-e^2, e^2].  scaled: [batch, T, d] reals of the component type; logscale: NULL or [batch, T]
 * reals receiving c (-inf for a zero state, whose scaled entries are 0).  Arguments otherwise as
 * for goom_affine_scan.  For GOOM_C64 with d = 16 or 32 and more than one chunk the last phase
 * writes the scaled states directly and no GOOM states touch memory; otherwise they pass through
 * the workspace.  workspace: goom_affine_scan_scaled_workspace_bytes(...) bytes. */
int goom_affine_scan_scaled(goom_ctx *ctx, const void *A, const void *bias, const void *h0,
                            void *scaled, void *logscale, int64_t T, int d, int64_t batch,
                            int dtype, const goom_scan_opts *opts, void *workspace,
                            size_t workspace_bytes);
size_t goom_affine_scan_scaled_workspace_bytes(int64_t T, int d, int64_t batch, int dtype,
                                               const goom_scan_opts *opts);

/* ---- backward passes (paper Section 3.1, the redefined finite derivatives; Section 3.2, log-scaling constants
 *      take no part in gradients; Section 4.3) ------------------------------------------------------------ */

/* Backward of goom_to_goom with respect to the log-magnitudes: the logarithm of a real x is log(abs(x)) with
 * d abs(x) / dx := +1 for x >= 0, -1 for x < 0 (never zero; paper eq. 5) and d log(u) / du := 1 / (u + eps)
 * (always finite; eq. 6), so grad_x[i] = grad_re[i] * s(x[i]) / (|x[i]| + eps).  x, grad_re, grad_x: n reals of
 * the component type (grad_re: gradient with respect to Re y[i]; the phase is piecewise constant and takes no
 * gradient).  eps >= 0: the paper's data-type-specific small number, left to the caller. */
int goom_to_goom_backward(goom_ctx *ctx, const void *x, const void *grad_re, void *grad_x, size_t n, int dtype,
                          double eps);

/* Backward of goom_from_goom: x = Re exp(y) with d exp(y) / dy := exp(y) + eps for x >= 0, exp(y) - eps for
 * x < 0 (never zero; paper eq. 8), so grad_re[i] = grad_x[i] * (x[i] + s(x[i]) eps), the gradient with respect
 * to Re y[i].  y: n GOOMs; grad_x, grad_re: n reals of the component type. */
int goom_from_goom_backward(goom_ctx *ctx, const void *y, const void *grad_x, void *grad_re, size_t n, int dtype,
                            double eps);

/* Backward of goom_scaled_exp and of the scaled states of goom_affine_scan_scaled (paper Section 4.3): the log-scaling
 * constant c = max Re z is computed without altering gradients, so scaled[i] = +-exp(Re z[i] - c + 2) has
 * d scaled[i] / d Re z[i] = scaled[i], also for the entry that sets c: grad_re[i] = grad_scaled[i] * scaled[i].
 * scaled (as returned by the forward call), grad_scaled, grad_re: n reals of the component type (device). */
int goom_scaled_exp_backward(goom_ctx *ctx, const void *scaled, const void *grad_scaled, void *grad_re, size_t n,
                             int dtype);

/* Backward of goom_lmme (paper Section 3.2 with the derivatives of Section 3.1 in the limit eps -> 0, as for the
 * recurrence below).  With C = A B over reals and grad_C[b, i, k] = dL / d Re C'[b, i, k] for some loss L,
 *     grad_A[b, i, j] = dL / d Re A'[b, i, j] = A_ij sum_k (grad_C_ik / C_ik) B_jk,
 *     grad_B[b, j, k] = dL / d Re B'[b, j, k] = B_jk sum_i A_ij (grad_C_ik / C_ik),
 * two products of the same kind, taken over GOOMs by the forward LMME on operands with the row maxima of A' and the
 * column maxima of B' (as whole numbers) taken out, so that log-magnitudes far from zero lose nothing to the
 * component type.  An entry of C that is exactly zero passes no gradient, nor does a zero entry of grad_C.
 * A: [batch, n, d], B: [batch, d, m], C: [batch, n, m] GOOMs as given to and returned by goom_lmme; grad_C:
 * [batch, n, m], grad_A: [batch, n, d], grad_B: [batch, d, m] reals of the component type (device, caller-owned;
 * grad_A and grad_B overwritten).  Sizes and flags as for goom_lmme (flags go to both products).  workspace:
 * goom_lmme_backward_workspace_bytes(...) bytes, required: about (n m + 2 n d + 2 d m) GOOMs per batch item
 * (n m for n = d = m = 128 without GOOM_LMME_EXACT, where the product kernel transposes and exponentiates itself).
 * Errors: GOOM_EINVAL (null or misaligned pointers, sizes), GOOM_EUNSUPPORTED (sizes beyond goom_lmme's),
 * GOOM_EWORKSPACE. */
int goom_lmme_backward(goom_ctx *ctx, const void *A, const void *B, const void *C, const void *grad_C, void *grad_A,
                       void *grad_B, int64_t batch, int n, int d, int m, int dtype, uint32_t flags, void *workspace,
                       size_t workspace_bytes);
size_t goom_lmme_backward_workspace_bytes(int64_t batch, int n, int d, int m, int dtype, uint32_t flags);

/* Backward of goom_scan (paper Section 4.1 with the derivatives of Section 3.1 in the limit eps -> 0).  With
 * P_t = M_t P_{t-1}, P_{-1} = S0 (the identity without one), and grad_P[b, t, i, k] = dL / d Re P[b, t, i, k],
 * the adjoints of the state values, Lam_t = grad_P_t / P_t + M_{t+1}^T Lam_{t+1} (d x m matrices), are the upper
 * block of a prefix scan of stacked (d + m) x (d + m) matrices [[M_{t+1}^T, grad_P_t / P_t], [0, I]] in reverse
 * time, run by goom_scan itself on log-magnitudes shifted to ordinary size, and
 *     grad_M[b, t, i, j] = M_t[i, j] sum_k Lam_t[i, k] P_{t-1}[j, k],    grad_S0[b, j, k] = S0[j, k] (M_0^T Lam_0)[j, k]
 * (one batched LMME).  A state entry that is exactly zero passes no gradient.
 * M: [batch, T, d, d], S0: NULL or [batch, d, m], P: [batch, T, d, m] GOOMs as given to and returned by goom_scan
 * (m = d without S0); grad_P: [batch, T, d, m], grad_M: [batch, T, d, d], grad_S0: NULL or [batch, d, m] (needs
 * S0) reals of the component type; device, caller-owned, outputs overwritten.  d + m <= GOOM_MAX_DIM_LMME.
 * opts: as for goom_scan (chunk length of the reverse scan); flags must be 0.  workspace:
 * goom_scan_backward_workspace_bytes(..., with_init = S0 != NULL) bytes, required: about
 * (d + m)(d + 2 m) GOOMs per step.  Errors: GOOM_EINVAL, GOOM_EUNSUPPORTED (sizes), GOOM_EWORKSPACE. */
int goom_scan_backward(goom_ctx *ctx, const void *M, const void *S0, const void *P, const void *grad_P, void *grad_M,
                       void *grad_S0, int64_t T, int d, int m, int64_t batch, int dtype, const goom_scan_opts *opts,
                       void *workspace, size_t workspace_bytes);
size_t goom_scan_backward_workspace_bytes(int64_t T, int d, int m, int64_t batch, int dtype,
                                          const goom_scan_opts *opts, int with_init);

/* Backward of goom_affine_scan (time-varying matrices).  grad_H[b, t, i] = dL / d Re H[b, t, i] for some loss L;
 * the call returns dL / d Re A[b, t, i, j], dL / d Re bias[b, t, i] and dL / d Re h0[b, j], as reals of the
 * component type.  The adjoints of the state values, lam_t = grad_H_t / h_t + A_{t+1}^T lam_{t+1}, are a
 * recurrence of the same kind in reverse time over the transposed matrices; they are computed over GOOMs by the
 * forward scan on transposed, time-reversed operands (they shrink as fast as the states grow), and
 *     grad_A[b, t, i, j] = lam_t[i] A_t[i, j] h_{t-1}[j],      grad_bias[b, t, i] = lam_t[i] b_t[i],
 *     grad_h0[b, j] = h0[j] sum_i lam_0[i] A_0[i, j].
 * This is the limit eps -> 0 of the paper's redefined derivatives, which differ from the ordinary ones only where
 * a value lies within eps of zero; a state entry that is exactly zero passes no gradient.
 * A, bias, h0 (NULL = zero), H: as given to and returned by goom_affine_scan; grad_H: [batch, T, d] reals;
 * grad_A: [batch, T, d, d] reals; grad_bias: NULL or [batch, T, d] reals; grad_h0: NULL or [batch, d] reals (needs
 * h0).  opts->flags: 0, or GOOM_AFFINE_TIME_INVARIANT for the recurrence with one matrix per batch item (the paper's
 * state-space layer, Section 4.3): A and grad_A are [batch, d, d], grad_A[b, i, j] = A[i, j] sum_t lam_t[i] h_{t-1}[j],
 * summed in double in a fixed order.  workspace: goom_affine_scan_backward_workspace_bytes(...) bytes: a few vectors per
 * step for complex64 with d = 16 or 32 and more than one chunk (the scan reads A transposed itself); otherwise it
 * also holds a transposed copy of A and is a little larger than A. */
int goom_affine_scan_backward(goom_ctx *ctx, const void *A, const void *bias, const void *h0, const void *H,
                              const void *grad_H, void *grad_A, void *grad_bias, void *grad_h0, int64_t T, int d,
                              int64_t batch, int dtype, const goom_scan_opts *opts, void *workspace,
                              size_t workspace_bytes);
size_t goom_affine_scan_backward_workspace_bytes(int64_t T, int d, int64_t batch, int dtype,
                                                 const goom_scan_opts *opts);

#pragma GCC visibility pop
#ifdef __cplusplus
}
#endif
#endif /* GOOM_H */
