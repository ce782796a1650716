/*
 * rsvd.h - C ABI of the MI355X (gfx950) randomized SVD library.
 *
 * The library computes the randomized k-SVD of the paper's Algorithm 1:
 * given A (m x n), a target rank k, an oversampling p, a power-scheme
 * exponent q and a seed, it returns the k largest singular values S and the
 * matching singular vectors U (m x k) and V^T (k x n) of the rank-k
 * approximation A_k ~ U diag(S) V^T.  With s = k + p (called l below):
 *   step 1  Omega (n x l) Gaussian sketch
 *   step 2  Y = (A A^T)^q A Omega, re-orthonormalised after every product
 *   step 3  Q = orthonormal basis of range(Y)
 *   step 4  B = Q^T A (l x n)          (held as B^T = A^T Q, n x l)
 *   step 5  B = Ub Sigma V^T           (one-sided Jacobi on the l x l factor)
 *   step 6  U = Q Ub[:, :k]
 *
 * Conventions for every entry point
 *   - All matrix pointers are DEVICE pointers to row-major storage with a
 *     leading dimension in elements; fp32 or fp64 as named by rsvd_dtype.
 *     Pointers must be aligned to the element size; 16-byte alignment of
 *     base pointers and leading dimensions enables the vector load paths.
 *   - The caller owns every buffer.  The library allocates no device memory
 *     in any of these calls; scratch comes from the caller's `workspace`
 *     (device memory, 256-byte aligned, at least rsvd_workspace_bytes()).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls are asynchronous on that stream unless stated otherwise.
 *   - A (and every input) is read-only and never modified.
 *   - Return value: 0 success; -i the i-th argument (1-based, counting as in
 *     the prototype) is invalid; positive values are rsvd_status codes.
 *   - Singular values are descending; signs of singular vectors are not
 *     normalised (u_i, v_i may both flip).
 *   - Calls that share a workspace, or a context, must not overlap in time.
 */
#ifndef RSVD_H
#define RSVD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rsvd_ctx rsvd_ctx;

typedef enum { RSVD_F32 = 0, RSVD_F64 = 1 } rsvd_dtype;

/* Which outputs to produce.  The paper's values-only mode stops after step 5
 * (remark after the step notes); step 6 is done "if required". */
typedef enum { RSVD_JOB_S = 0, RSVD_JOB_SV = 1, RSVD_JOB_SUV = 2 } rsvd_job;

typedef enum {
  RSVD_OK = 0,
  RSVD_ERR_NONFINITE = 1,   /* a Gram matrix held a non-finite entry (non-finite input) */
  RSVD_ERR_NO_CONVERGENCE = 2, /* Jacobi did not converge within the sweep cap */
  RSVD_ERR_HIP = 3,         /* a HIP runtime call failed; see rsvd_last_hip_error */
  RSVD_ERR_UNSUPPORTED = 4, /* shape outside what the kernels support (l too large) */
  RSVD_ERR_NO_DEVICE = 5,   /* the context was created with RSVD_DEVICE_NONE: it can size and check, not run */
  RSVD_ERR_SCRATCH_LIMIT = 6 /* rsvd_run_static: the problem needs more than RSVD_STATIC_SCRATCH_BYTES of workspace */
} rsvd_status;

/* Diagnostics written by rsvd_run / stage calls when the caller asks for them
 * (host memory; filling it forces a stream synchronisation). */
typedef struct {
  int32_t status;          /* rsvd_status accumulated on the device */
  int32_t jacobi_sweeps;   /* sweeps the small SVD used */
  int32_t refilled_columns;/* columns found linearly dependent and replaced by
                              fresh Gaussian directions, summed over all
                              orthonormalisations of the call.  A column counts
                              as dependent when what is left of it after the
                              earlier columns is below the resolution of the
                              orthonormalisation: ~4e-6 of its norm for fp32
                              data (the rounding level of the panel itself),
                              ~1e-12 for fp64 data */
  int32_t skipped_reorth;   /* 1: the condition estimate of the first panel let the power scheme drop one of
                             * its two re-orthonormalisations per iteration (see rsvd_run); else 0 */
  int32_t raised_pivots;    /* fp64 only: pivots that fell below the resolution of one CholeskyQR round
                             * (~1e-6 of the column norm) and were carried into an additional round instead of
                             * being dropped, summed over the call.  Non-zero says that the sketched spectrum
                             * spans more than six decades; it costs one more round per orthonormalisation */
} rsvd_info;

/* Create / destroy a context for HIP device `device`.  Host-side only:
 * queries device properties, allocates nothing on the device.  The calls
 * below launch on the caller's stream and never switch devices: that device
 * must be the current one when they are made.
 * device = RSVD_DEVICE_NONE gives a planning context that makes no HIP call at
 * all (a scheduler or a build machine without a GPU can size workspaces and
 * validate arguments with it): the workspace queries answer for an MI355X,
 * every other call checks its arguments as usual and then returns
 * RSVD_ERR_NO_DEVICE instead of launching. */
#define RSVD_DEVICE_NONE (-1)
int rsvd_create(rsvd_ctx **ctx, int device);
int rsvd_destroy(rsvd_ctx *ctx);

const char *rsvd_status_string(int code);
/* Text of the last HIP error seen by this context (host string, owned by ctx). */
const char *rsvd_last_hip_error(const rsvd_ctx *ctx);

/* Per-kernel timing for benchmarks (host-side state of the context; off by
 * default).  While enabled, every kernel launch of every call on this context
 * is bracketed by a pair of HIP events on the call's stream.
 * rsvd_profile_read waits for the recorded events, sums elapsed milliseconds
 * and launch counts per kernel class into total_ms / launches (host arrays of
 * n_kinds >= 12 entries, index = class; names from rsvd_profile_kind_name)
 * and clears the record. */
int rsvd_profile_enable(rsvd_ctx *ctx, int on);
int rsvd_profile_read(rsvd_ctx *ctx, int n_kinds, double *total_ms, int *launches);
const char *rsvd_profile_kind_name(int kind);

/* Bytes of device workspace that rsvd_run and every stage call need for a
 * problem of this size (one figure covers all of them). */
int rsvd_workspace_bytes(rsvd_ctx *ctx, rsvd_dtype dtype, int64_t m, int64_t n,
                         int k, int p, int q, rsvd_job job, size_t *bytes);

/*
 * Algorithm 1, all six steps.
 *   A      m x n, leading dimension lda >= n
 *   S      k values (device)
 *   U      m x k, leading dimension ldu >= k   (RSVD_JOB_SUV, else may be NULL)
 *   Vt     k x n, leading dimension ldvt >= n  (RSVD_JOB_SV / SUV, else may be NULL)
 *   info   host pointer or NULL.  Non-NULL: the call synchronises `stream`
 *          before returning and the return value includes device-side status.
 *          NULL: the call only enqueues kernels on `stream` - no allocation,
 *          no synchronisation, no memset nodes, nothing read from the
 *          workspace before it is written - so it may be recorded into a HIP
 *          graph (after one ordinary call of the same shape) and replayed.
 * Singular values that are numerically zero (below eps * ||B||_F, B = Q^T A):
 * their rows of Vt are orthonormal like all the others, their columns of U are
 * zero (the small SVD rotates the rows of the triangular factor of B^T and
 * normalises what is left of them; nothing is left of these).
 * Requires k >= 1, p >= 0, q >= 0, k + p <= min(m, n).
 * Re-orthonormalisation inside the power scheme (step 2; the algorithm as
 * printed has none, it is there for floating point): after every product by
 * default.  When the triangular factor of the first panel A Omega shows a
 * small condition number (estimate ||R||_F ||R^-1||_F / sqrt(k + p) at most
 * 32 in fp32, 128 in fp64), one of the two factorisations of every iteration
 * is dropped - decided on the device, no synchronisation; info->skipped_reorth
 * reports it.  The basis of step 3 always gets its full treatment.
 */
int rsvd_run(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, rsvd_job job,
             int64_t m, int64_t n, const void *A, int64_t lda,
             int k, int p, int q, uint64_t seed,
             void *S, void *U, int64_t ldu, void *Vt, int64_t ldvt,
             void *workspace, size_t workspace_bytes, rsvd_info *info);

/*
 * rsvd_run for callers that cannot allocate device memory and have no workspace
 * to hand over: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same computation, same kernels and same results as
 * rsvd_run (bit for bit); the workspace is a buffer of
 * RSVD_STATIC_SCRATCH_BYTES (32 MiB) that lives inside the loaded library, one
 * copy per GPU, held until the process ends.  The call allocates nothing and
 * frees nothing (with per-kernel profiling off, its default).
 *   - A problem whose rsvd_workspace_bytes() exceeds the buffer is turned away
 *     with RSVD_ERR_SCRATCH_LIMIT before anything is launched (the paper's
 *     10000 x 2000, k + p = 80 benchmark shape needs 29 MiB and fits).
 *   - Every call on one GPU uses the same buffer, whatever the context or the
 *     stream: calls that overlap in time on one GPU race.  The buffer keeps the
 *     contents of the call before; the kernels clear what they need cleared.
 *   - info as for rsvd_run (non-NULL synchronises the stream).
 * Arguments 1-17 as rsvd_run.  rsvd_static_scratch_bytes() returns the limit.
 */
#define RSVD_STATIC_SCRATCH_BYTES (32u << 20)
int rsvd_run_static(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, rsvd_job job,
                    int64_t m, int64_t n, const void *A, int64_t lda,
                    int k, int p, int q, uint64_t seed,
                    void *S, void *U, int64_t ldu, void *Vt, int64_t ldvt, rsvd_info *info);
size_t rsvd_static_scratch_bytes(void);

/*
 * The paper's PCA application: the same decomposition of the column-centred
 * matrix A - 1 mu^T (mu = column means of A, rows = observations), computed
 * without forming that matrix: the product kernels take mu_j (kept in fp64)
 * away from every element of A while they stage it, so the result is as
 * accurate as on a matrix centred beforehand, however large the means are
 * against the spread of the data.  S^2 / (m - 1) are the
 * variances along the principal axes, the rows of Vt the axes, U diag(S) the
 * scores.  Arguments as rsvd_run, positions 1-20 unchanged; `mean` (device,
 * n values, may be NULL) receives mu.
 */
int rsvd_run_centered(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, rsvd_job job,
                      int64_t m, int64_t n, const void *A, int64_t lda,
                      int k, int p, int q, uint64_t seed,
                      void *S, void *U, int64_t ldu, void *Vt, int64_t ldvt,
                      void *workspace, size_t workspace_bytes, rsvd_info *info, void *mean);

/*
 * Many small problems at once (the paper's clustering application calls the
 * solver on a great number of data blocks): `batch` matrices of one shape,
 * problem b at A + b * stride_a elements, its results at S + b * stride_s,
 * U + b * stride_u and Vt + b * stride_vt.  Every kernel launch of Algorithm 1
 * covers the whole batch, so the single-workgroup steps (Cholesky, Jacobi) of
 * different problems run side by side.  Problem b draws its sketch with
 * seed + b; its results equal those of rsvd_run on that matrix with that seed
 * up to the rounding of a different split of the long sums.
 *   requires k + p <= 128, the reach of the single-workgroup kernels
 *   (RSVD_ERR_UNSUPPORTED otherwise; fp64 problems beyond 96 accumulate the
 *   rotations of step 5 in global memory and take about twice as long there),
 *   batch in 1 .. 65535, strides that
 *   keep the problems apart, and a workspace of rsvd_workspace_bytes_batched().
 *   info (host, may be NULL) describes the whole batch: the worst status, the
 *   largest sweep count, the total of replaced columns.
 */
int rsvd_workspace_bytes_batched(rsvd_ctx *ctx, rsvd_dtype dtype, int batch, int64_t m, int64_t n,
                                 int k, int p, int q, rsvd_job job, size_t *bytes);
int rsvd_run_batched(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, rsvd_job job, int batch,
                     int64_t m, int64_t n, const void *A, int64_t lda, int64_t stride_a,
                     int k, int p, int q, uint64_t seed,
                     void *S, int64_t stride_s, void *U, int64_t ldu, int64_t stride_u,
                     void *Vt, int64_t ldvt, int64_t stride_vt,
                     void *workspace, size_t workspace_bytes, rsvd_info *info);

/* ---- stage entry points: each step of Algorithm 1 on its own, for per-stage
 * parity tests and timing.  They run the same kernels as rsvd_run. ---- */

/* Bytes of workspace that the stage calls which work on one rows x l panel need (rsvd_stage_orth and
 * rsvd_stage_small_svd with that panel; rsvd_stage_jacobi with rows = l): the panels and l x l matrices only,
 * nothing sized by a matrix A.  The figure of rsvd_workspace_bytes() for an m x n problem with m, n >= rows and
 * the same k + p = l also suffices; the product stages (rsvd_stage_gemm_an / _atn) take that figure. */
int rsvd_stage_workspace_bytes(rsvd_ctx *ctx, rsvd_dtype dtype, int64_t rows, int64_t l, size_t *bytes);

/* Step 1: Omega (rows x cols, leading dimension ldo) of iid N(0,1) from
 * Philox4x32-10 + Box-Muller; element (i, j) is element i*cols + j of stream
 * `stream_id` under `seed` (stream 0 is the sketch of rsvd_run). */
int rsvd_stage_sketch(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype,
                      uint64_t seed, uint32_t stream_id, int64_t rows, int64_t cols,
                      void *Omega, int64_t ldo);

/* Debug hook for bit-exact parity of the generator: raw Philox4x32-10 outputs
 * for counter groups first_group .. first_group + n_groups - 1, written as
 * 4 x uint32 per group to `out` (device). */
int rsvd_stage_philox_raw(rsvd_ctx *ctx, void *stream, uint64_t seed, uint32_t stream_id,
                          uint64_t first_group, int64_t n_groups, uint32_t *out);

/* Steps 2 and 6: Y (m x l) = A (m x n) X (n x l). */
int rsvd_stage_gemm_an(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype,
                       int64_t m, int64_t n, int64_t l,
                       const void *A, int64_t lda, const void *X, int64_t ldx,
                       void *Y, int64_t ldy, void *workspace, size_t workspace_bytes);

/* Power scheme and step 4: Z (n x l) = A^T (n x m) X (m x l), A given as m x n. */
int rsvd_stage_gemm_atn(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype,
                        int64_t m, int64_t n, int64_t l,
                        const void *A, int64_t lda, const void *X, int64_t ldx,
                        void *Z, int64_t ldz, void *workspace, size_t workspace_bytes);

/* Step 3: replace Y (rows x l, leading dimension ldy, in place) by Q with
 * orthonormal columns and range(Q) containing range(Y) (CholeskyQR, two
 * rounds, Gram matrix accumulated and factored in fp64).  A column that is
 * numerically dependent on the ones before it is replaced by a fresh Gaussian
 * direction (Philox stream `refill_stream`), so Q always has l orthonormal
 * columns.  R (l x l, fp64, ld l, device, may be NULL) receives the upper
 * triangular factor with Y = Q R (rows of replaced columns are zero). */
int rsvd_stage_orth(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype,
                    int64_t rows, int64_t l, void *Y, int64_t ldy, double *R,
                    uint64_t seed, uint32_t refill_stream,
                    void *workspace, size_t workspace_bytes, rsvd_info *info);

/* Step 5 on the transposed factor: Bt (n x l, leading dimension ldbt) holds
 * B^T.  Outputs (device, all l triplets, sigma descending):
 *   sigma (l), Ub (l x l, ld l) left singular vectors of B,
 *   V (n x l, leading dimension ldv) right singular vectors of B as columns.
 * B = Ub diag(sigma) V^T.  Bt is overwritten. */
int rsvd_stage_small_svd(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype,
                         int64_t n, int64_t l, void *Bt, int64_t ldbt,
                         void *sigma, void *Ub, void *V, int64_t ldv,
                         uint64_t seed, void *workspace, size_t workspace_bytes,
                         rsvd_info *info);

/* One-sided Jacobi SVD of a small square matrix alone: M (l x l, ld l, row-major,
 * overwritten) = X diag(sigma) W^T; sigma descending, X and W l x l (ld l).
 * The rotations act on the columns of M (W accumulates them and is orthogonal
 * to rounding whatever M is; a column of X that belongs to a numerically zero
 * singular value is zero).  They converge in the fewest sweeps when the columns
 * are graded in length, as the rows of a triangular factor are: for such an M
 * pass its transpose and swap X and W (rsvd_run and rsvd_stage_small_svd do
 * that with the factor of B^T).  RSVD_ERR_NO_CONVERGENCE after 60 sweeps
 * (24 above the single-workgroup orders). */
int rsvd_stage_jacobi(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, int64_t l,
                      void *M, void *sigma, void *X, void *W,
                      void *workspace, size_t workspace_bytes, rsvd_info *info);

/* Step 6: U (m x k, leading dimension ldu) = Q (m x l) W[:, :k] (W l x l, ld ldw).
 * With transpose_out != 0 the product is stored transposed (k x m, leading
 * dimension ldu >= m), which is how V^T is produced. */
int rsvd_stage_lift(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype,
                    int64_t m, int64_t l, int64_t k,
                    const void *Q, int64_t ldq, const void *W, int64_t ldw,
                    void *U, int64_t ldu, int transpose_out,
                    void *workspace, size_t workspace_bytes);

#ifdef __cplusplus
}
#endif
#endif /* RSVD_H */
