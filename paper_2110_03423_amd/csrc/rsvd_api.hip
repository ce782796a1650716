// C ABI of the library: argument checks, workspace layout and the sequence of
// kernel launches for Algorithm 1 (sketch, range product, power scheme with
// re-orthonormalisation, projection, small SVD, lift).  Host code only.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <new>

#include "common.hpp"

namespace rsvd {

size_t gemm_partial_bytes_f32(const rsvd_ctx *, int64_t, int64_t, int64_t, int);
size_t gemm_partial_bytes_f64(const rsvd_ctx *, int64_t, int64_t, int64_t, int);
size_t gemm_partial_bytes_f32acc64(const rsvd_ctx *, int64_t, int64_t, int64_t, int);
hipError_t gemm_launch_f32(rsvd_ctx *, hipStream_t, const GemmDesc &);
hipError_t gemm_launch_f64(rsvd_ctx *, hipStream_t, const GemmDesc &);
hipError_t gemm_launch_f32acc64(rsvd_ctx *, hipStream_t, const GemmDesc &);

size_t gemm_partial_bytes(const rsvd_ctx *ctx, GemmKind kind, int trans_a, int64_t M, int64_t N, int64_t K) {
  switch (kind) {
    case GEMM_F32: return gemm_partial_bytes_f32(ctx, M, N, K, trans_a);
    case GEMM_F64: return gemm_partial_bytes_f64(ctx, M, N, K, trans_a);
    default:       return gemm_partial_bytes_f32acc64(ctx, M, N, K, trans_a);
  }
}

hipError_t gemm_launch(rsvd_ctx *ctx, hipStream_t s, GemmKind kind, const GemmDesc &d) {
  switch (kind) {
    case GEMM_F32: return gemm_launch_f32(ctx, s, d);
    case GEMM_F64: return gemm_launch_f64(ctx, s, d);
    default:       return gemm_launch_f32acc64(ctx, s, d);
  }
}

// skip_flag (device int, stride_flag bytes between the problems of a batch; may be NULL): non-zero = do nothing
template <typename T>
__global__ void copy_kernel(const T *__restrict__ src, T *__restrict__ dst, int64_t n, int64_t stride_src,
                            int64_t stride_dst, const int *skip_flag, int64_t stride_flag) {
  if (skip_flag != nullptr &&
      *reinterpret_cast<const int *>(reinterpret_cast<const char *>(skip_flag) + (int64_t)blockIdx.y * stride_flag) != 0)
    return;
  src = reinterpret_cast<const T *>(reinterpret_cast<const char *>(src) + (int64_t)blockIdx.y * stride_src);
  dst = reinterpret_cast<T *>(reinterpret_cast<char *>(dst) + (int64_t)blockIdx.y * stride_dst);
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x)
    dst[e] = src[e];
}

// rows x cols elements from src (leading dimension lds) to dst (leading dimension ldd); one problem.
template <typename T>
__global__ __launch_bounds__(256) void copy2d_kernel(const T *__restrict__ src, int64_t lds, T *__restrict__ dst,
                                                     int64_t ldd, int64_t rows, int64_t cols, const int *skip_flag) {
  if (skip_flag != nullptr && *skip_flag != 0) return;
  const int64_t total = rows * cols;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = e / cols, c = e - r * cols;
    dst[r * ldd + c] = src[r * lds + c];
  }
}

// Column means: out64[j] = (1 / rows) * sum_i X[i][j], accumulated in fp64 in two deterministic
// stages (row chunks of kColsumRows, then the chunks in order); out (may be NULL) receives the
// same values rounded to the matrix type.
constexpr int kColsumRows = 512;

template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T *__restrict__ X, int64_t ldx, int64_t rows,
                                                             int64_t cols, double *__restrict__ partial) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t r0 = (int64_t)blockIdx.y * kColsumRows;
  const int64_t r1 = (r0 + kColsumRows < rows) ? r0 + kColsumRows : rows;
  if (j >= cols) return;
  // eight independent partial sums keep eight loads in flight
  double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  int64_t i = r0;
  for (; i + 8 <= r1; i += 8) {
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] += (double)X[(i + u) * ldx + j];
  }
  for (; i < r1; ++i) acc[0] += (double)X[i * ldx + j];
  partial[(int64_t)blockIdx.y * cols + j] = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
}

template <typename T>
__global__ __launch_bounds__(256) void colsum_final_kernel(const double *__restrict__ partial, int chunks, int64_t cols,
                                                           double alpha, double *__restrict__ out64,
                                                           T *__restrict__ out) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= cols) return;
  double acc[4] = {0, 0, 0, 0};
  int c = 0;
  for (; c + 4 <= chunks; c += 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[u] += partial[(int64_t)(c + u) * cols + j];
  }
  for (; c < chunks; ++c) acc[0] += partial[(int64_t)c * cols + j];
  const double mu = alpha * ((acc[0] + acc[1]) + (acc[2] + acc[3]));
  out64[j] = mu;
  if (out != nullptr) out[j] = (T)mu;
}

static size_t colsum_partial_bytes(int64_t rows, int64_t cols) {
  return (size_t)ceil_div(rows, kColsumRows) * (size_t)cols * sizeof(double);
}

static hipError_t colmean_launch(hipStream_t s, rsvd_dtype dtype, const void *X, int64_t ldx, int64_t rows,
                                 int64_t cols, double *out64, void *out, void *partial, size_t partial_bytes) {
  const int chunks = (int)ceil_div(rows, kColsumRows);
  if (partial == nullptr || partial_bytes < colsum_partial_bytes(rows, cols)) return hipErrorInvalidValue;
  dim3 grid((unsigned)ceil_div(cols, 256), (unsigned)chunks);
  dim3 grid2((unsigned)ceil_div(cols, 256));
  const double alpha = 1.0 / (double)rows;
  if (dtype == RSVD_F32) {
    hipLaunchKernelGGL(colsum_partial_kernel<float>, grid, dim3(256), 0, s, (const float *)X, ldx, rows, cols,
                       (double *)partial);
    hipLaunchKernelGGL(colsum_final_kernel<float>, grid2, dim3(256), 0, s, (const double *)partial, chunks, cols,
                       alpha, out64, (float *)out);
  } else {
    hipLaunchKernelGGL(colsum_partial_kernel<double>, grid, dim3(256), 0, s, (const double *)X, ldx, rows, cols,
                       (double *)partial);
    hipLaunchKernelGGL(colsum_final_kernel<double>, grid2, dim3(256), 0, s, (const double *)partial, chunks, cols,
                       alpha, out64, (double *)out);
  }
  return hipGetLastError();
}

// batch > 1: problem b copies from src + b * stride_src to dst + b * stride_dst (bytes)
static hipError_t copy_launch(hipStream_t s, rsvd_dtype dtype, const void *src, void *dst, int64_t n, int batch = 1,
                              int64_t stride_src = 0, int64_t stride_dst = 0, const int *skip_flag = nullptr) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = ceil_div(n, 256);
  if (blocks > 4096) blocks = 4096;
  const dim3 grid((unsigned)blocks, (unsigned)batch);
  // (a gate lives in the workspace of its problem: same stride as the workspace buffers)
  if (dtype == RSVD_F32)
    hipLaunchKernelGGL(copy_kernel<float>, grid, dim3(256), 0, s, (const float *)src, (float *)dst, n, stride_src,
                       stride_dst, skip_flag, stride_src);
  else
    hipLaunchKernelGGL(copy_kernel<double>, grid, dim3(256), 0, s, (const double *)src, (double *)dst, n, stride_src,
                       stride_dst, skip_flag, stride_src);
  return hipGetLastError();
}

static hipError_t copy2d_launch(hipStream_t s, rsvd_dtype dtype, const void *src, int64_t lds, void *dst, int64_t ldd,
                                int64_t rows, int64_t cols, const int *skip_flag) {
  int64_t blocks = ceil_div(rows * cols, 256 * 8);
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  if (dtype == RSVD_F32)
    hipLaunchKernelGGL(copy2d_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, s, (const float *)src, lds,
                       (float *)dst, ldd, rows, cols, skip_flag);
  else
    hipLaunchKernelGGL(copy2d_kernel<double>, dim3((unsigned)blocks), dim3(256), 0, s, (const double *)src, lds,
                       (double *)dst, ldd, rows, cols, skip_flag);
  return hipGetLastError();
}

__global__ void widen_kernel(const float *__restrict__ src, double *__restrict__ dst, int64_t n) {
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x)
    dst[e] = (double)src[e];
}

static hipError_t widen_launch(hipStream_t s, const float *src, double *dst, int64_t n) {
  hipLaunchKernelGGL(widen_kernel, dim3(256), dim3(256), 0, s, src, dst, n);
  return hipGetLastError();
}

// ---------------------------------------------------------------- workspace

// Offsets (bytes) into the caller's workspace.  Depends on (dtype, m, n, l) only.
struct Layout {
  size_t bufM[2], bufN[2];          // m x l and n x l panels (ld l), ping-pong for CholeskyQR
  size_t partial, partial_bytes;    // split-K scratch
  size_t G, chol_scratch;           // fp64 Gram matrix, blocked-Cholesky scratch
  size_t Rinv, R1, R2, R3, R4, Rb;  // R^-1 (dtype), R factors of the rounds and their product (fp64)
  size_t dead, info;                // flags per column, DevInfo
  size_t flags;                     // device-side switches (ints): [0] = the power scheme may skip one side,
                                    // [1], [2] = no pivot was raised in the first / second CholeskyQR round:
                                    // the additional round that would resolve it is skipped
  size_t sigma, Wj, Xj;             // all l triplets of step 5: sigma, Ub (= W), X
  size_t jac_scratch, jac_scratch_bytes;
  size_t mean;                      // centred variant: column means (n, fp64)
  size_t total;
};

static Layout make_layout(const rsvd_ctx *ctx, rsvd_dtype dtype, int64_t m, int64_t n, int64_t l) {
  Layout L;
  const size_t es = dtype_size(dtype);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  for (int i = 0; i < 2; ++i) L.bufM[i] = take((size_t)m * l * es);
  for (int i = 0; i < 2; ++i) L.bufN[i] = take((size_t)n * l * es);
  const GemmKind kind = dtype == RSVD_F32 ? GEMM_F32 : GEMM_F64;
  const GemmKind gram = dtype == RSVD_F32 ? GEMM_F32_ACC64 : GEMM_F64;
  size_t pb = gemm_partial_bytes(ctx, kind, 0, m, l, n);
  size_t t;
  if ((t = gemm_partial_bytes(ctx, kind, 1, n, l, m)) > pb) pb = t;
  if ((t = gemm_partial_bytes(ctx, gram, 1, l, l, m)) > pb) pb = t;
  if ((t = gemm_partial_bytes(ctx, gram, 1, l, l, n)) > pb) pb = t;
  if ((t = gram_syrk_partial_bytes(ctx, m, l)) > pb) pb = t;
  if ((t = gram_syrk_partial_bytes(ctx, n, l)) > pb) pb = t;
  if ((t = colsum_partial_bytes(m, n)) > pb) pb = t;      // column means of the centred variant
  L.partial_bytes = pb;
  L.partial = take(pb);
  L.G = take((size_t)l * l * 8);
  L.chol_scratch = take(chol_scratch_elems(ctx, l) * 8);
  L.Rinv = take((size_t)l * l * es);
  L.R1 = take((size_t)l * l * 8);
  L.R2 = take((size_t)l * l * 8);
  L.R3 = take(dtype == RSVD_F64 ? (size_t)l * l * 8 : 0);      // the additional rounds exist for fp64 panels only
  L.R4 = take(dtype == RSVD_F64 ? (size_t)l * l * 8 : 0);
  L.Rb = take((size_t)l * l * 8);
  L.dead = take((size_t)l * sizeof(int));
  L.info = take(sizeof(DevInfo));
  L.flags = take(16 * sizeof(int));
  L.sigma = take((size_t)l * es);
  L.Wj = take((size_t)l * l * es);
  L.Xj = take((size_t)l * l * es);
  L.jac_scratch_bytes = jacobi_scratch_bytes(ctx, dtype, l);
  L.jac_scratch = take(L.jac_scratch_bytes);
  L.mean = take((size_t)n * 8);
  L.total = off;
  return L;
}

struct Ws {
  char *base;
  Layout L;
  int batch = 1;           // equal-shaped problems handled by every launch
  int64_t stride = 0;      // bytes between the workspaces of consecutive problems (every buffer of L)
  template <typename P> P *at(size_t off) const { return reinterpret_cast<P *>(base + off); }
};

static int fail_hip(rsvd_ctx *ctx, hipError_t e, const char *where) {
  snprintf(ctx->hip_error, sizeof(ctx->hip_error), "%s: %s", where, hipGetErrorString(e));
  return RSVD_ERR_HIP;
}

#define RSVD_TRY(expr, where)                                   \
  do {                                                          \
    hipError_t e_ = (expr);                                     \
    if (e_ != hipSuccess) return fail_hip(ctx, e_, where);      \
  } while (0)

// ---------------------------------------------------------------- building blocks

// Y (rows x l, ld ldy) -> Q by `rounds` (1 or 2) rounds of CholeskyQR; `tmp` is a
// rows x l panel (ld l).  Two rounds leave Q in Y with columns orthonormal to
// working precision.  One round leaves it in `tmp`: a well-conditioned basis of
// the same range (orthonormal to about cond(Y) * eps), which is all the power
// scheme needs between two products.  Rout (fp64, l x l, two rounds only)
// receives R with Y = Q R, or NULL.
// skip_flag (device int, or NULL): when it reads non-zero every launch of this call does nothing (the caller then
// goes on with Y itself).  keep_r: the triangular factor of the first round is also written to the R1 buffer.
//
// Resolution.  The Gram matrix is held in fp64, so a first round separates directions of Y down to sqrt(tau) ~ 1e-6
// of the largest one; what lies below drowns in the rounding of the Gram matrix.  For fp32 panels that is the
// end of it (the panel itself carries nothing finer) and such a column is replaced by a fresh Gaussian
// direction.  For fp64 panels - where Householder QR, the paper's step 3, would keep directions down to the
// rounding level of the data - such a column is SET ASIDE instead (see chol.hip): it stays in the panel, divided by
// sqrt(threshold) and so short of unit length, the round sets a device flag, and AN ADDITIONAL ROUND, issued with every call and
// switched on by that flag, works on a panel whose weak directions have been magnified by 1 / sqrt(tau).  Each
// round resolves another six decades; a two-round call has two additional rounds behind it and so reaches the
// rounding level of the data, a one-round call (inside the power scheme) one, which keeps ~1e-12.  Only what is
// below that (or exactly zero) is replaced.  Without raised pivots the additional rounds return at once and the
// result is the one of the plain scheme, bit for bit.
static int orthonormalize(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype dtype, const Ws &w, int64_t rows, int64_t l,
                          void *Y, int64_t ldy, void *tmp, double *Rout, uint64_t seed, uint32_t refill_stream,
                          int rounds = 2, const int *skip_flag = nullptr, bool keep_r = false) {
  const GemmKind kind = dtype == RSVD_F32 ? GEMM_F32 : GEMM_F64;
  const GemmKind gram = dtype == RSVD_F32 ? GEMM_F32_ACC64 : GEMM_F64;
  const Layout &L = w.L;
  // pivot threshold (on squared norms): the rounding level of the fp64 Gram matrix and its elimination - and, for
  // fp32 panels, the rounding level of the panel itself: a column that is a product in fp32 carries noise of
  // ~1e-6 of its norm, and what is left of it below that after the earlier columns is that noise, not a
  // direction.  Kept as one, it is blown up by 1e6 in the triangular solve, and a second round no longer brings
  // the basis to working precision (seen as a reconstruction error of 400 eps on an exactly rank-deficient input).
  double tau = 32.0 * 2.220446049250313e-16 * ((double)l + sqrt((double)rows));
  if (dtype == RSVD_F32) {
    const double rel = 32.0 * 1.1920929e-07;           // 3.8e-6 of the column norm
    if (rel * rel > tau) tau = rel * rel;
  }
  const bool rescue = dtype == RSVD_F64;
  int *redo_skip = rescue ? w.at<int>(L.flags) + 1 : nullptr;      // 0 = the first round raised a pivot
  void *src = Y; int64_t lds_ = ldy;
  void *dst = tmp; int64_t ldd = l;
  // One round: Gram matrix of `from`, its factor, `to` = `from` R^-1 (`to` may be `from` when one tile row of the
  // product kernel spans all l columns: a workgroup has then read its rows completely before it writes them).
  auto one_round = [&](int round, const void *from, int64_t ld_from, void *to, int64_t ld_to, const int *gate,
                       const CholPivoting &pv, double *R) -> int {
    // Gram matrix: up to 128 columns the kernel that reads the panel once; beyond, the general product on the
    // upper tiles.  Up to four partial sums are left for the Cholesky kernel to add.
    int parts = 1;
    if (l <= gram_syrk_max_order()) {
      RSVD_TRY(gram_syrk_launch(ctx, s, dtype, rows, l, from, ld_from, w.at<double>(L.G), w.at<void>(L.partial),
                                L.partial_bytes, 4, &parts, w.batch, w.stride, gate),
               "gram");
    } else {
      GemmDesc g;
      g.trans_a = 1; g.M = l; g.N = l; g.K = rows;
      g.A = from; g.lda = ld_from; g.B = from; g.ldb = ld_from;
      g.C = w.at<double>(L.G); g.ldc = l;
      g.partial = w.at<void>(L.partial); g.partial_bytes = L.partial_bytes;
      g.prof_kind = PK_GRAM;
      g.batch = w.batch; g.stride_a = g.stride_b = g.stride_c = g.stride_partial = w.stride;
      g.skip_flag = gate; g.stride_flag = w.stride;
      g.upper_only = 1;              // the blocked factorisation reads the upper block triangle only
      RSVD_TRY(gemm_launch(ctx, s, gram, g), "gram");
    }
    RSVD_TRY(chol_inverse_launch(ctx, s, dtype, l, parts > 1 ? w.at<double>(L.partial) : w.at<double>(L.G), l, parts,
                                 l * l, tau, w.at<void>(L.Rinv), R, w.at<int>(L.dead), w.at<DevInfo>(L.info),
                                 w.at<double>(L.chol_scratch), w.batch, w.stride, gate, pv),
             "cholesky");
    if (l <= apply_tri_max_order(dtype)) {
      RSVD_TRY(apply_tri_launch(ctx, s, dtype, rows, l, from, ld_from, w.at<void>(L.Rinv), to, ld_to, w.at<int>(L.dead),
                                seed, refill_stream + (uint32_t)round, 1.0 / sqrt((double)rows), l, w.batch, w.stride,
                                gate),
               "apply R^-1");
      return 0;
    }
    GemmDesc a;
    a.M = rows; a.N = l; a.K = l;
    a.A = from; a.lda = ld_from; a.B = w.at<void>(L.Rinv); a.ldb = l;
    a.b_upper = 1;
    a.C = to; a.ldc = ld_to;
    a.dead = w.at<int>(L.dead); a.seed = seed; a.refill_stream = refill_stream + (uint32_t)round;
    a.refill_scale = 1.0 / sqrt((double)rows); a.refill_ld = l;
    a.force_splits = 1;
    a.batch = w.batch; a.stride_a = a.stride_b = a.stride_c = a.stride_dead = w.stride; a.seed_step = 1;
    a.skip_flag = gate; a.stride_flag = w.stride;
    a.prof_kind = PK_APPLY;
    RSVD_TRY(gemm_launch(ctx, s, kind, a), "apply R^-1");
    return 0;
  };
  // fp64 panels.  A column set aside in round r leaves it scaled by 1 / sqrt(tau), and so does the rounding noise
  // of the panel (~eps of a column of Y): behind r such rounds a column whose squared norm is below
  // (16 eps)^2 / tau^r holds nothing but that noise and is dropped.  From the second round on the resolved columns
  // have unit length and the pivot threshold is tau itself for every column.
  const double noise2 = 256.0 * 2.220446049250313e-16 * 2.220446049250313e-16;
  const double floor_after[3] = {0.0, noise2 / tau, noise2 / (tau * tau)};
  int *redo2_skip = redo_skip ? redo_skip + 1 : nullptr;             // 0 = the second round raised a pivot as well
  int rc;
  for (int round = 0; round < rounds; ++round) {
    CholPivoting pv;
    if (rescue) {
      // the first round of every call, and the second round of a two-round call (which then has a fourth to fall
      // back on), raise weak pivots; each leaves the switch of the additional round that resolves them
      pv.raise = 1;
      pv.redo_skip = round == 0 ? redo_skip : redo2_skip;
      if (round > 0) { pv.floor_abs = floor_after[round]; pv.abs_thr = tau; }
    }
    double *R = (Rout || (keep_r && round == 0)) ? w.at<double>(round == 0 ? L.R1 : L.R2) : nullptr;
    if ((rc = one_round(round, src, lds_, dst, ldd, skip_flag, pv, R))) return rc;
    void *tp = src; src = dst; dst = tp;
    int64_t tl = lds_; lds_ = ldd; ldd = tl;
  }
  // The additional rounds on the result (now in `src`): one behind a single round (the power scheme needs a
  // well-conditioned basis, not every last direction), two behind a double round; each runs when the round two
  // places before it raised a pivot.  Six decades of the panel's spectrum are resolved per round, so three
  // resolving rounds and a polishing one reach the rounding level of fp64; what is still weak in the last
  // resolving round is dropped and replaced.
  const int extra = rescue ? rounds : 0;
  for (int x = 0; x < extra; ++x) {
    const int *gate = x == 0 ? redo_skip : redo2_skip;
    CholPivoting pv;
    pv.abs_thr = tau;
    pv.floor_abs = rounds + x < 3 ? floor_after[rounds + x] : 0.0;      // (the fourth round sees unit columns only)
    double *R = Rout ? w.at<double>(x == 0 ? L.R3 : L.R4) : nullptr;
    if (l <= 128) {
      if ((rc = one_round(rounds + x, src, lds_, src, lds_, gate, pv, R))) return rc;
    } else {
      if ((rc = one_round(rounds + x, src, lds_, dst, ldd, gate, pv, R))) return rc;
      ProfScope ps(ctx, s, PK_SMALL);
      RSVD_TRY(copy2d_launch(s, dtype, dst, ldd, src, lds_, rows, l, gate), "copy panel");
    }
  }
  if (Rout) {
    ProfScope ps(ctx, s, PK_SMALL);
    RSVD_TRY(triu_product_launch(s, l, w.at<double>(L.R2), w.at<double>(L.R1), Rout, w.batch, w.stride), "R product");
    for (int x = 0; x < extra; ++x) {
      // R = R3 (R2 R1), then R4 (R3 R2 R1), for the additional rounds that ran
      const int *gate = x == 0 ? redo_skip : redo2_skip;
      RSVD_TRY(triu_product_launch(s, l, w.at<double>(x == 0 ? L.R3 : L.R4), Rout, w.at<double>(L.G), w.batch,
                                   w.stride, gate),
               "R product");
      RSVD_TRY(copy_launch(s, RSVD_F64, w.at<void>(L.G), Rout, l * l, w.batch, w.stride, w.stride, gate), "copy R");
    }
  }
  return 0;
}

static int product(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype dtype, const Ws &w, int trans_a, int64_t M, int64_t N,
                   int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb, void *C, int64_t ldc,
                   int trans_c, bool allow_split, int prof_kind, double alpha = 1.0, const double *a_shift = nullptr,
                   int64_t stride_a = -1, int64_t stride_c = -1, const int *alt_flag = nullptr,
                   const void *B_alt = nullptr) {
  // batched: B is always a workspace buffer; A and C are too unless the caller names their strides (bytes)
  GemmDesc d;
  d.batch = w.batch;
  d.stride_a = stride_a >= 0 ? stride_a : w.stride;
  d.stride_b = w.stride;
  d.stride_c = stride_c >= 0 ? stride_c : w.stride;
  d.stride_partial = w.stride;
  d.alt_flag = alt_flag; d.B_alt = B_alt; d.stride_flag = w.stride;      // *alt_flag != 0: B_alt is the operand
  d.prof_kind = prof_kind;
  d.alpha = alpha; d.a_shift = a_shift;
  d.trans_a = trans_a; d.trans_c = trans_c; d.M = M; d.N = N; d.K = K;
  d.A = A; d.lda = lda; d.B = B; d.ldb = ldb; d.C = C; d.ldc = ldc;
  if (allow_split) { d.partial = w.at<void>(w.L.partial); d.partial_bytes = w.L.partial_bytes; }
  else d.force_splits = 1;
  RSVD_TRY(gemm_launch(ctx, s, dtype == RSVD_F32 ? GEMM_F32 : GEMM_F64, d), "gemm");
  return 0;
}

// Step 5 on Bt (n x l, ld ldbt): Bt = Qb Rb, Rb = X Sigma W^T.  On exit Bt holds Qb,
// and sigma / W / X sit in the workspace.
static int small_svd(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype dtype, const Ws &w, int64_t n, int64_t l, void *Bt,
                     int64_t ldbt, void *tmp, uint64_t seed, uint32_t refill_stream) {
  const Layout &L = w.L;
  int rc = orthonormalize(ctx, s, dtype, w, n, l, Bt, ldbt, tmp, w.at<double>(L.Rb), seed, refill_stream);
  if (rc) return rc;
  // Rb = X Sigma W^T from the rows of Rb, i.e. from Rb^T = W Sigma X^T (hence the swapped outputs): the rows of the
  // triangular factor are graded like the singular values, its columns are not, and the rotations converge in
  // about half the sweeps on the former when the spectrum is steep (a third when the factor is rank deficient)
  hipError_t e = jacobi_launch(ctx, s, dtype, l, w.at<void>(L.Rb), 1, w.at<void>(L.sigma), w.at<void>(L.Wj),
                               w.at<void>(L.Xj), w.at<DevInfo>(L.info), w.at<void>(L.jac_scratch),
                               L.jac_scratch_bytes, w.batch, w.stride, 1);
  if (e == hipErrorNotSupported) return RSVD_ERR_UNSUPPORTED;
  RSVD_TRY(e, "jacobi");
  return 0;
}

static int finish_info(rsvd_ctx *ctx, hipStream_t s, const Ws &w, rsvd_info *info) {
  if (info == nullptr) return 0;
  DevInfo h;
  RSVD_TRY(hipMemcpyAsync(&h, w.at<DevInfo>(w.L.info), sizeof(h), hipMemcpyDeviceToHost, s), "info copy");
  RSVD_TRY(hipStreamSynchronize(s), "synchronize");
  info->status = h.status;
  info->jacobi_sweeps = h.jacobi_sweeps;
  info->refilled_columns = h.refilled;
  info->skipped_reorth = h.skipped_reorth;
  info->raised_pivots = h.raised;
  return h.status;
}

static bool valid_dtype(rsvd_dtype d) { return d == RSVD_F32 || d == RSVD_F64; }

}  // namespace rsvd

// Workspace of rsvd_run_static: device memory that belongs to the loaded library, one copy per GPU, held until
// the process ends.  The name is a host-side handle only; its device address is looked up once per context
// (hipGetSymbolAddress, in rsvd_create) and that address is what the kernels receive.
constexpr size_t kStaticScratchBytes = (size_t)RSVD_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

using namespace rsvd;

extern "C" {

int rsvd_create(rsvd_ctx **out, int device) {
  if (out == nullptr) return -1;
  *out = nullptr;
  // RSVD_DEVICE_NONE: a planning context with the MI355X's figures, touching no HIP call
  hipDeviceProp_t prop;
  memset(&prop, 0, sizeof(prop));
  if (device == RSVD_DEVICE_NONE) {
    prop.multiProcessorCount = 256;
    prop.sharedMemPerBlock = 160 * 1024;
  } else if (device < 0 || hipGetDeviceProperties(&prop, device) != hipSuccess) {
    return -2;
  }
  rsvd_ctx *c = new (std::nothrow) rsvd_ctx;
  if (c == nullptr) return RSVD_ERR_HIP;
  c->device = device;
  c->cu_count = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  size_t lds = prop.sharedMemPerBlock;
#if HIP_VERSION_MAJOR >= 6
  if (prop.sharedMemPerBlockOptin > lds) lds = prop.sharedMemPerBlockOptin;
#endif
  if (lds > 160 * 1024) lds = 160 * 1024;
  if (lds < 32 * 1024) lds = 32 * 1024;
  c->lds_per_block = lds;
  c->hip_error[0] = 0;
  c->prof_on = false;
  c->prof_used = 0;
  c->static_scratch = nullptr;
  if (device >= 0) {
    // address of this device's copy of the static scratch array (the device must be current for the lookup)
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e == hipSuccess && cur != device) e = hipSetDevice(device);
    if (e == hipSuccess) {
      void *ptr = nullptr;
      e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (e == hipSuccess) c->static_scratch = ptr;
      else snprintf(c->hip_error, sizeof(c->hip_error), "static scratch lookup: %s", hipGetErrorString(e));
      // per-kernel launch limits (dynamic LDS) of the single-workgroup kernels, for this device
      hipError_t e2 = chol_init_device(c);
      if (e2 == hipSuccess) e2 = jacobi_init_device(c);
      if (e2 == hipSuccess) e2 = apply_init_device(c);
      if (e2 == hipSuccess) e2 = gram_init_device(c);
      if (cur >= 0 && cur != device) (void)hipSetDevice(cur);
      if (e2 != hipSuccess) {
        (void)hipGetLastError();
        delete c;
        return RSVD_ERR_HIP;
      }
    }
    if (e != hipSuccess) (void)hipGetLastError();
  }
  *out = c;
  return 0;
}

int rsvd_destroy(rsvd_ctx *ctx) {
  if (ctx != nullptr)
    for (hipEvent_t e : ctx->prof_events) (void)hipEventDestroy(e);
  delete ctx;
  return 0;
}

const char *rsvd_status_string(int code) {
  switch (code) {
    case RSVD_OK: return "success";
    case RSVD_ERR_NONFINITE: return "non-finite values met during orthonormalisation";
    case RSVD_ERR_NO_CONVERGENCE: return "Jacobi SVD did not converge within the sweep cap";
    case RSVD_ERR_HIP: return "HIP runtime error";
    case RSVD_ERR_UNSUPPORTED: return "problem shape not supported";
    case RSVD_ERR_NO_DEVICE: return "planning context (RSVD_DEVICE_NONE): arguments are valid, nothing was launched";
    case RSVD_ERR_SCRATCH_LIMIT: return "problem needs more workspace than the static scratch buffer of rsvd_run_static holds";
    default: return code < 0 ? "invalid argument" : "unknown status";
  }
}

const char *rsvd_last_hip_error(const rsvd_ctx *ctx) { return ctx ? ctx->hip_error : ""; }

int rsvd_profile_enable(rsvd_ctx *ctx, int on) {
  if (ctx == nullptr) return -1;
  ctx->prof_on = on != 0;
  ctx->prof_used = 0;
  return 0;
}

const char *rsvd_profile_kind_name(int kind) {
  static const char *names[PK_COUNT] = {"sketch", "gemm_ax", "gemm_ax_reduce", "gemm_atx", "gemm_atx_reduce",
                                        "gram", "gram_reduce", "cholesky", "apply_rinv", "jacobi", "lift", "small"};
  return (kind >= 0 && kind < PK_COUNT) ? names[kind] : "?";
}

int rsvd_profile_read(rsvd_ctx *ctx, int n_kinds, double *total_ms, int *launches) {
  if (ctx == nullptr) return -1;
  if (n_kinds < PK_COUNT) return -2;
  if (total_ms == nullptr) return -3;
  if (launches == nullptr) return -4;
  for (int i = 0; i < n_kinds; ++i) { total_ms[i] = 0.0; launches[i] = 0; }
  for (size_t i = 0; i < ctx->prof_used; ++i) {
    float ms = 0.f;
    RSVD_TRY(hipEventSynchronize(ctx->prof_events[2 * i + 1]), "event sync");
    RSVD_TRY(hipEventElapsedTime(&ms, ctx->prof_events[2 * i], ctx->prof_events[2 * i + 1]), "event time");
    total_ms[ctx->prof_kinds[i]] += ms;
    launches[ctx->prof_kinds[i]] += 1;
  }
  ctx->prof_used = 0;
  return 0;
}

int rsvd_workspace_bytes(rsvd_ctx *ctx, rsvd_dtype dtype, int64_t m, int64_t n, int k, int p, int q, rsvd_job job,
                         size_t *bytes) {
  if (ctx == nullptr) return -1;
  if (!valid_dtype(dtype)) return -2;
  if (m < 1) return -3;
  if (n < 1) return -4;
  if (k < 1) return -5;
  if (p < 0 || (int64_t)k + p > (m < n ? m : n)) return -6;
  if (q < 0) return -7;
  if (job < RSVD_JOB_S || job > RSVD_JOB_SUV) return -8;
  if (bytes == nullptr) return -9;
  *bytes = make_layout(ctx, dtype, m, n, (int64_t)k + p).total;
  return 0;
}

// Algorithm 1 on A, or (center != 0) on A - 1 mu^T with mu the column means of A, without forming that matrix:
// the product kernels take mu_j (fp64) away from every element of A on its way into LDS, so the result carries
// rounding errors of the size of the centred entries, not of the means.
// batch > 1: `batch` problems of the same shape, problem b at A + b * stride_a elements (likewise S, U, Vt), sketch
// seed + b; every kernel launch covers the whole batch.  Needs l within the single-workgroup Cholesky and Jacobi
// kernels and no centring; the diagnostics are those of the whole batch (worst status, most sweeps, all replaced
// columns).
static int run_impl(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, rsvd_job job, int64_t m, int64_t n, const void *A,
                    int64_t lda, int k, int p, int q, uint64_t seed, void *S, void *U, int64_t ldu, void *Vt,
                    int64_t ldvt, void *workspace, size_t workspace_bytes, rsvd_info *info, int center,
                    void *mean_out, int batch = 1, int64_t stride_a = 0, int64_t stride_s = 0, int64_t stride_u = 0,
                    int64_t stride_vt = 0) {
  if (ctx == nullptr) return -1;
  if (!valid_dtype(dtype)) return -3;
  if (job < RSVD_JOB_S || job > RSVD_JOB_SUV) return -4;
  if (m < 1) return -5;
  if (n < 1) return -6;
  if (A == nullptr) return -7;
  if (lda < n) return -8;
  if (k < 1) return -9;
  if (p < 0 || (int64_t)k + p > (m < n ? m : n)) return -10;
  if (q < 0) return -11;
  if (S == nullptr) return -13;
  if (job == RSVD_JOB_SUV && U == nullptr) return -14;
  if (job == RSVD_JOB_SUV && ldu < k) return -15;
  if (job >= RSVD_JOB_SV && Vt == nullptr) return -16;
  if (job >= RSVD_JOB_SV && ldvt < n) return -17;
  const int64_t l = (int64_t)k + p;
  const int64_t es = (int64_t)dtype_size(dtype);
  Ws w;
  w.L = make_layout(ctx, dtype, m, n, l);
  w.base = (char *)workspace;
  w.batch = batch;
  w.stride = (int64_t)w.L.total;             // a multiple of 256
  if (workspace == nullptr || ((uintptr_t)workspace & 255) != 0) return -18;
  if (workspace_bytes < w.L.total * (size_t)batch) return -19;
  if (l > jacobi_max_lds_order(ctx, dtype) && jacobi_scratch_bytes(ctx, dtype, l) == 0) return RSVD_ERR_UNSUPPORTED;
  if (batch > 1 && (l > jacobi_max_batched_order(ctx, dtype) || l > chol_max_block(ctx) || center))
    return RSVD_ERR_UNSUPPORTED;
  if (ctx->device < 0) return RSVD_ERR_NO_DEVICE;
  hipStream_t s = (hipStream_t)stream;
  const Layout &L = w.L;
  void *bM0 = w.at<void>(L.bufM[0]), *bM1 = w.at<void>(L.bufM[1]);
  void *bN0 = w.at<void>(L.bufN[0]), *bN1 = w.at<void>(L.bufN[1]);
  int rc;

  RSVD_TRY(zero_ints_launch(s, w.at<int>(L.info), kDevInfoInts), "zero info");
  double *mean = center ? w.at<double>(L.mean) : nullptr;
  if (center) {
    // mu = A^T 1 / m, kept in fp64 for the products and handed out in the matrix type
    ProfScope ps(ctx, s, PK_SMALL);
    RSVD_TRY(colmean_launch(s, dtype, A, lda, m, n, mean, mean_out, w.at<void>(L.partial), L.partial_bytes), "means");
  }
  // products with the (optionally centred) matrix; X is n x l for A X, m x l for A^T X
  // (alt_flag / X_alt: when the device flag reads non-zero, X_alt is multiplied instead of X)
  auto times_a = [&](const void *X, void *Y, const int *alt_flag = nullptr, const void *X_alt = nullptr) -> int {
    return product(ctx, s, dtype, w, 0, m, l, n, A, lda, X, l, Y, l, 0, true, PK_GEMM_AX, 1.0, mean, stride_a * es, -1,
                   alt_flag, X_alt);
  };
  auto times_at = [&](const void *X, void *Z, const int *alt_flag = nullptr, const void *X_alt = nullptr) -> int {
    return product(ctx, s, dtype, w, 1, n, l, m, A, lda, X, l, Z, l, 0, true, PK_GEMM_ATX, 1.0, mean, stride_a * es, -1,
                   alt_flag, X_alt);
  };
  // step 1
  {
    ProfScope ps(ctx, s, PK_SKETCH);
    RSVD_TRY(sketch_launch(s, dtype, seed, 0u, n, l, bN0, l, batch, w.stride), "sketch");
  }
  // step 2: Y = A Omega, then q rounds of Z = A^T Q, Y = A Z.  Every product is
  // re-orthonormalised; all but the last with a single CholeskyQR round (result in
  // the other panel of the pair), the last one (step 3) with two.
  //
  // Adaptive schedule (Algorithm 1 as printed has no factorisation inside the power scheme at all; the
  // re-orthonormalisation is there for floating point): the factor R of the first panel Y = A Omega gives an
  // upper bound kappa_F = ||R||_F ||R^-1||_F of its condition number, which is that of A on the sketched range.
  // A panel that is multiplied by A (or A^T) without being orthonormalised first arrives with that number squared,
  // so when kappa_F is small enough for the precision, one of the two orthonormalisations of every iteration
  // is switched off ON THE DEVICE (flag in the workspace; the launches are still issued and return at once, the
  // next product reads the raw panel).  The side that is dropped is the more expensive one; the final basis
  // (step 3) always gets its two rounds.
  void *curN = bN0, *othN = bN1, *curM = bM0, *othM = bM1;
  uint32_t refill = 16;
  auto swap = [](void *&a, void *&b) { void *t = a; a = b; b = t; };
  const bool adaptive = q > 0;
  const int *skip = adaptive ? w.at<int>(L.flags) : nullptr;
  const bool drop_m = adaptive && (int64_t)(q - 1) * m > (int64_t)q * n;      // else the n-side ones are dropped
  if ((rc = times_a(curN, curM))) return rc;
  if ((rc = orthonormalize(ctx, s, dtype, w, m, l, curM, l, othM, nullptr, seed, refill, q == 0 ? 2 : 1, nullptr,
                           adaptive)))
    return rc;
  if (adaptive) {
    // kappa_F overestimates the 2-norm condition number by a factor between 1 and l (about sqrt(l) for the
    // decaying and the noise-floor spectra met here), so kappa_F / sqrt(l) serves as the estimate.  A skipped
    // factorisation costs about eps * kappa^2 in the weakest sketched direction, and the next Gram matrix has
    // condition kappa^4, which must stay clear of the dependent-column threshold: estimate <= 32 (fp32), 128 (fp64).
    ProfScope ps(ctx, s, PK_SMALL);
    const double limit = (dtype == RSVD_F32 ? 32.0 : 128.0) * sqrt((double)l);
    RSVD_TRY(cond_flag_launch(s, dtype, l, w.at<double>(L.R1), w.at<void>(L.Rinv), limit, w.at<int>(L.flags),
                              w.at<DevInfo>(L.info), batch, w.stride,
                              dtype == RSVD_F64 ? w.at<int>(L.flags) + 1 : nullptr),
             "condition flag");
  }
  if (q > 0) swap(curM, othM);
  refill += 3;
  bool m_raw = false;          // the previous m-side factorisation may have been skipped: raw panel in othM
  for (int it = 0; it < q; ++it) {
    if ((rc = times_at(curM, curN, m_raw ? skip : nullptr, m_raw ? othM : nullptr))) return rc;
    const bool n_skippable = adaptive && !drop_m;
    if ((rc = orthonormalize(ctx, s, dtype, w, n, l, curN, l, othN, nullptr, seed, refill, 1,
                             n_skippable ? skip : nullptr)))
      return rc;
    swap(curN, othN);
    refill += 3;
    if ((rc = times_a(curN, curM, n_skippable ? skip : nullptr, n_skippable ? othN : nullptr))) return rc;
    const bool last = it == q - 1;
    m_raw = adaptive && drop_m && !last;
    if ((rc = orthonormalize(ctx, s, dtype, w, m, l, curM, l, othM, nullptr, seed, refill, last ? 2 : 1,
                             m_raw ? skip : nullptr)))
      return rc;
    if (!last) swap(curM, othM);
    refill += 3;
  }
  // step 4: B^T = A^T Q
  if ((rc = times_at(curM, curN))) return rc;
  // step 5
  if ((rc = small_svd(ctx, s, dtype, w, n, l, curN, l, othN, seed, refill))) return rc;
  RSVD_TRY(copy_launch(s, dtype, w.at<void>(L.sigma), S, k, batch, w.stride, stride_s * es), "copy S");
  if (job >= RSVD_JOB_SV) {
    // V^T = (Qb X[:, :k])^T
    if ((rc = product(ctx, s, dtype, w, 0, n, k, l, curN, l, w.at<void>(L.Xj), l, Vt, ldvt, 1, false, PK_LIFT, 1.0,
                      nullptr, -1, stride_vt * es)))
      return rc;
  }
  if (job == RSVD_JOB_SUV) {
    // step 6: U = Q Ub[:, :k]
    if ((rc = product(ctx, s, dtype, w, 0, m, k, l, curM, l, w.at<void>(L.Wj), l, U, ldu, 0, false, PK_LIFT, 1.0,
                      nullptr, -1, stride_u * es)))
      return rc;
  }
  return finish_info(ctx, s, w, info);
}

int rsvd_run(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, rsvd_job job, int64_t m, int64_t n, const void *A,
             int64_t lda, int k, int p, int q, uint64_t seed, void *S, void *U, int64_t ldu, void *Vt, int64_t ldvt,
             void *workspace, size_t workspace_bytes, rsvd_info *info) {
  return run_impl(ctx, stream, dtype, job, m, n, A, lda, k, p, q, seed, S, U, ldu, Vt, ldvt, workspace,
                  workspace_bytes, info, 0, nullptr);
}

int rsvd_stage_workspace_bytes(rsvd_ctx *ctx, rsvd_dtype dtype, int64_t rows, int64_t l, size_t *bytes) {
  if (ctx == nullptr) return -1;
  if (!valid_dtype(dtype)) return -2;
  if (rows < 1) return -3;
  if (l < 1 || l > rows) return -4;
  if (bytes == nullptr) return -5;
  *bytes = make_layout(ctx, dtype, rows, l, l).total;
  return 0;
}

int rsvd_run_static(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, rsvd_job job, int64_t m, int64_t n, const void *A,
                    int64_t lda, int k, int p, int q, uint64_t seed, void *S, void *U, int64_t ldu, void *Vt,
                    int64_t ldvt, rsvd_info *info) {
  if (ctx == nullptr) return -1;
  // size check first (host arithmetic only), so that an oversized problem is turned away before anything else
  size_t need = 0;
  if (valid_dtype(dtype) && m >= 1 && n >= 1 && k >= 1 && p >= 0 && (int64_t)k + p <= (m < n ? m : n)) {
    need = make_layout(ctx, dtype, m, n, (int64_t)k + p).total;
    if (need > kStaticScratchBytes) return RSVD_ERR_SCRATCH_LIMIT;
  }
  void *ws = ctx->static_scratch;
  if (ctx->device < 0) ws = reinterpret_cast<void *>((uintptr_t)256);      // planning context: checked, never used
  if (ws == nullptr) {
    if (ctx->hip_error[0] == 0) snprintf(ctx->hip_error, sizeof(ctx->hip_error), "static scratch is not available");
    return RSVD_ERR_HIP;
  }
  return run_impl(ctx, stream, dtype, job, m, n, A, lda, k, p, q, seed, S, U, ldu, Vt, ldvt, ws, kStaticScratchBytes,
                  info, 0, nullptr);
}

size_t rsvd_static_scratch_bytes(void) { return kStaticScratchBytes; }

int rsvd_run_centered(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, rsvd_job job, int64_t m, int64_t n,
                      const void *A, int64_t lda, int k, int p, int q, uint64_t seed, void *S, void *U, int64_t ldu,
                      void *Vt, int64_t ldvt, void *workspace, size_t workspace_bytes, rsvd_info *info, void *mean) {
  return run_impl(ctx, stream, dtype, job, m, n, A, lda, k, p, q, seed, S, U, ldu, Vt, ldvt, workspace,
                  workspace_bytes, info, 1, mean);
}

int rsvd_workspace_bytes_batched(rsvd_ctx *ctx, rsvd_dtype dtype, int batch, int64_t m, int64_t n, int k, int p,
                                 int q, rsvd_job job, size_t *bytes) {
  if (batch < 1 || batch > 65535) return -3;
  size_t one = 0;
  const int rc = rsvd_workspace_bytes(ctx, dtype, m, n, k, p, q, job, &one);
  if (rc != 0) return rc < -2 ? rc - 1 : rc;          // arguments after `batch` sit one place later here
  if (bytes == nullptr) return -10;
  *bytes = one * (size_t)batch;
  return 0;
}

int rsvd_run_batched(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, rsvd_job job, int batch, int64_t m, int64_t n,
                     const void *A, int64_t lda, int64_t stride_a, int k, int p, int q, uint64_t seed, void *S,
                     int64_t stride_s, void *U, int64_t ldu, int64_t stride_u, void *Vt, int64_t ldvt,
                     int64_t stride_vt, void *workspace, size_t workspace_bytes, rsvd_info *info) {
  if (batch < 1 || batch > 65535) return -5;
  // positions of the arguments in this prototype (run_impl reports those of rsvd_run)
  static const int pos[20] = {0, 1, 2, 3, 4, 6, 7, 8, 9, 11, 12, 13, 14, 15, 17, 18, 20, 21, 23, 24};
  if (batch > 1) {
    if (stride_a < (m - 1) * lda + n) return -10;
    if (stride_s < k) return -16;
    if (job == RSVD_JOB_SUV && stride_u < (m - 1) * ldu + k) return -19;
    if (job >= RSVD_JOB_SV && stride_vt < (int64_t)(k - 1) * ldvt + n) return -22;
  }
  const int rc = run_impl(ctx, stream, dtype, job, m, n, A, lda, k, p, q, seed, S, U, ldu, Vt, ldvt, workspace,
                          workspace_bytes, info, 0, nullptr, batch, stride_a, stride_s, stride_u, stride_vt);
  return (rc < 0 && -rc < 20) ? -pos[-rc] : rc;
}

int rsvd_stage_sketch(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, uint64_t seed, uint32_t stream_id, int64_t rows,
                      int64_t cols, void *Omega, int64_t ldo) {
  if (ctx == nullptr) return -1;
  if (!valid_dtype(dtype)) return -3;
  if (rows < 0) return -6;
  if (cols < 0) return -7;
  if (rows * cols == 0) return 0;
  if (Omega == nullptr) return -8;
  if (ldo < cols) return -9;
  if (ctx->device < 0) return RSVD_ERR_NO_DEVICE;
  RSVD_TRY(sketch_launch((hipStream_t)stream, dtype, seed, stream_id, rows, cols, Omega, ldo), "sketch");
  return 0;
}

int rsvd_stage_philox_raw(rsvd_ctx *ctx, void *stream, uint64_t seed, uint32_t stream_id, uint64_t first_group,
                          int64_t n_groups, uint32_t *out) {
  if (ctx == nullptr) return -1;
  if (n_groups < 0) return -6;
  if (n_groups == 0) return 0;
  if (out == nullptr) return -7;
  if (ctx->device < 0) return RSVD_ERR_NO_DEVICE;
  RSVD_TRY(philox_raw_launch((hipStream_t)stream, seed, stream_id, first_group, n_groups, out), "philox");
  return 0;
}

static int stage_gemm(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, int trans_a, int64_t m, int64_t n, int64_t l,
                      const void *A, int64_t lda, const void *X, int64_t ldx, void *Y, int64_t ldy, void *workspace,
                      size_t workspace_bytes) {
  if (ctx == nullptr) return -1;
  if (!valid_dtype(dtype)) return -3;
  if (m < 1) return -4;
  if (n < 1) return -5;
  if (l < 1 || l > (m < n ? m : n)) return -6;
  if (A == nullptr) return -7;
  if (lda < n) return -8;
  if (X == nullptr) return -9;
  if (ldx < l) return -10;
  if (Y == nullptr) return -11;
  if (ldy < l) return -12;
  Ws w;
  w.L = make_layout(ctx, dtype, m, n, l);
  w.base = (char *)workspace;
  if (workspace == nullptr || ((uintptr_t)workspace & 255) != 0) return -13;
  if (workspace_bytes < w.L.total) return -14;
  if (ctx->device < 0) return RSVD_ERR_NO_DEVICE;
  if (trans_a) return product(ctx, (hipStream_t)stream, dtype, w, 1, n, l, m, A, lda, X, ldx, Y, ldy, 0, true, PK_GEMM_ATX);
  return product(ctx, (hipStream_t)stream, dtype, w, 0, m, l, n, A, lda, X, ldx, Y, ldy, 0, true, PK_GEMM_AX);
}

int rsvd_stage_gemm_an(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, int64_t m, int64_t n, int64_t l, const void *A,
                       int64_t lda, const void *X, int64_t ldx, void *Y, int64_t ldy, void *workspace,
                       size_t workspace_bytes) {
  return stage_gemm(ctx, stream, dtype, 0, m, n, l, A, lda, X, ldx, Y, ldy, workspace, workspace_bytes);
}

int rsvd_stage_gemm_atn(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, int64_t m, int64_t n, int64_t l, const void *A,
                        int64_t lda, const void *X, int64_t ldx, void *Z, int64_t ldz, void *workspace,
                        size_t workspace_bytes) {
  return stage_gemm(ctx, stream, dtype, 1, m, n, l, A, lda, X, ldx, Z, ldz, workspace, workspace_bytes);
}

int rsvd_stage_orth(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, int64_t rows, int64_t l, void *Y, int64_t ldy,
                    double *R, uint64_t seed, uint32_t refill_stream, void *workspace, size_t workspace_bytes,
                    rsvd_info *info) {
  if (ctx == nullptr) return -1;
  if (!valid_dtype(dtype)) return -3;
  if (rows < 1) return -4;
  if (l < 1 || l > rows) return -5;
  if (Y == nullptr) return -6;
  if (ldy < l) return -7;
  Ws w;
  w.L = make_layout(ctx, dtype, rows, l, l);           // a rows x l panel and l x l matrices: nothing sized by a matrix A
  w.base = (char *)workspace;
  if (workspace == nullptr || ((uintptr_t)workspace & 255) != 0) return -11;
  if (workspace_bytes < w.L.total) return -12;
  if (ctx->device < 0) return RSVD_ERR_NO_DEVICE;
  hipStream_t s = (hipStream_t)stream;
  RSVD_TRY(zero_ints_launch(s, w.at<int>(w.L.info), kDevInfoInts), "zero info");
  int rc = orthonormalize(ctx, s, dtype, w, rows, l, Y, ldy, w.at<void>(w.L.bufM[1]),
                          R ? w.at<double>(w.L.Rb) : nullptr, seed, refill_stream);
  if (rc) return rc;
  if (R) RSVD_TRY(copy_launch(s, RSVD_F64, w.at<void>(w.L.Rb), R, l * l), "copy R");
  return finish_info(ctx, s, w, info);
}

int rsvd_stage_small_svd(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, int64_t n, int64_t l, void *Bt, int64_t ldbt,
                         void *sigma, void *Ub, void *V, int64_t ldv, uint64_t seed, void *workspace,
                         size_t workspace_bytes, rsvd_info *info) {
  if (ctx == nullptr) return -1;
  if (!valid_dtype(dtype)) return -3;
  if (n < 1) return -4;
  if (l < 1 || l > n) return -5;
  if (Bt == nullptr) return -6;
  if (ldbt < l) return -7;
  if (sigma == nullptr) return -8;
  if (Ub == nullptr) return -9;
  if (V == nullptr) return -10;
  if (ldv < l) return -11;
  Ws w;
  w.L = make_layout(ctx, dtype, n, l, l);              // as rsvd_stage_orth: the n x l panel takes the "m" slots
  w.base = (char *)workspace;
  if (workspace == nullptr || ((uintptr_t)workspace & 255) != 0) return -13;
  if (workspace_bytes < w.L.total) return -14;
  if (l > jacobi_max_lds_order(ctx, dtype) && jacobi_scratch_bytes(ctx, dtype, l) == 0) return RSVD_ERR_UNSUPPORTED;
  if (ctx->device < 0) return RSVD_ERR_NO_DEVICE;
  hipStream_t s = (hipStream_t)stream;
  RSVD_TRY(zero_ints_launch(s, w.at<int>(w.L.info), kDevInfoInts), "zero info");
  int rc = small_svd(ctx, s, dtype, w, n, l, Bt, ldbt, w.at<void>(w.L.bufM[1]), seed, 16u);
  if (rc) return rc;
  RSVD_TRY(copy_launch(s, dtype, w.at<void>(w.L.sigma), sigma, l), "copy sigma");
  RSVD_TRY(copy_launch(s, dtype, w.at<void>(w.L.Wj), Ub, l * l), "copy Ub");
  if ((rc = product(ctx, s, dtype, w, 0, n, l, l, Bt, ldbt, w.at<void>(w.L.Xj), l, V, ldv, 0, false, PK_LIFT))) return rc;
  return finish_info(ctx, s, w, info);
}

int rsvd_stage_jacobi(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, int64_t l, void *M, void *sigma, void *X, void *W,
                      void *workspace, size_t workspace_bytes, rsvd_info *info) {
  if (ctx == nullptr) return -1;
  if (!valid_dtype(dtype)) return -3;
  if (l < 1) return -4;
  if (M == nullptr) return -5;
  if (sigma == nullptr) return -6;
  if (X == nullptr) return -7;
  if (W == nullptr) return -8;
  Ws w;
  w.L = make_layout(ctx, dtype, l, l, l);
  w.base = (char *)workspace;
  if (workspace == nullptr || ((uintptr_t)workspace & 255) != 0) return -9;
  if (workspace_bytes < w.L.total) return -10;
  if (ctx->device < 0) return RSVD_ERR_NO_DEVICE;
  hipStream_t s = (hipStream_t)stream;
  RSVD_TRY(zero_ints_launch(s, w.at<int>(w.L.info), kDevInfoInts), "zero info");
  const void *Min = M;
  int min_f64 = dtype == RSVD_F64;
  if (dtype == RSVD_F32 && l > jacobi_max_lds_order(ctx, dtype)) {
    // the block path reads an fp64 matrix: widen M into the slot of the triangular factor
    RSVD_TRY(widen_launch(s, (const float *)M, w.at<double>(w.L.Rb), l * l), "widen");
    Min = w.at<void>(w.L.Rb);
    min_f64 = 1;
  }
  hipError_t e = jacobi_launch(ctx, s, dtype, l, Min, min_f64, sigma, X, W, w.at<DevInfo>(w.L.info),
                               w.at<void>(w.L.jac_scratch), w.L.jac_scratch_bytes);
  if (e == hipErrorNotSupported) return RSVD_ERR_UNSUPPORTED;
  RSVD_TRY(e, "jacobi");
  return finish_info(ctx, s, w, info);
}

int rsvd_stage_lift(rsvd_ctx *ctx, void *stream, rsvd_dtype dtype, int64_t m, int64_t l, int64_t k, const void *Q,
                    int64_t ldq, const void *W, int64_t ldw, void *U, int64_t ldu, int transpose_out, void *workspace,
                    size_t workspace_bytes) {
  (void)workspace; (void)workspace_bytes;
  if (ctx == nullptr) return -1;
  if (!valid_dtype(dtype)) return -3;
  if (m < 1) return -4;
  if (l < 1) return -5;
  if (k < 1 || k > l) return -6;
  if (Q == nullptr) return -7;
  if (ldq < l) return -8;
  if (W == nullptr) return -9;
  if (ldw < k) return -10;
  if (U == nullptr) return -11;
  if (ldu < (transpose_out ? m : k)) return -12;
  if (ctx->device < 0) return RSVD_ERR_NO_DEVICE;
  Ws w;
  w.base = nullptr;
  memset(&w.L, 0, sizeof(w.L));
  return product(ctx, (hipStream_t)stream, dtype, w, 0, m, k, l, Q, ldq, W, ldw, U, ldu, transpose_out ? 1 : 0, false, PK_LIFT);
}

}  // extern "C"
