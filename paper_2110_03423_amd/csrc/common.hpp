// Shared host-side declarations of the rSVD library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/rsvd.h"

struct rsvd_ctx {
  int device;
  int cu_count;
  size_t lds_per_block;     // bytes of LDS one workgroup may use
  char hip_error[256];
  // optional per-kernel timing (rsvd_profile_*): one event pair per launch
  bool prof_on;
  std::vector<hipEvent_t> prof_events;   // pairs: start, stop
  std::vector<int> prof_kinds;           // one per pair
  size_t prof_used;                      // pairs recorded since the last read
  void *static_scratch;                  // device address of this GPU's static scratch array (rsvd_run_static), or NULL
};

namespace rsvd {

constexpr int kWave = 64;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t dtype_size(rsvd_dtype d) { return d == RSVD_F32 ? 4 : 8; }

// Kernel classes reported by the profiling interface.
enum ProfKind {
  PK_SKETCH = 0, PK_GEMM_AX, PK_GEMM_AX_REDUCE, PK_GEMM_ATX, PK_GEMM_ATX_REDUCE, PK_GRAM, PK_GRAM_REDUCE,
  PK_CHOL, PK_APPLY, PK_JACOBI, PK_LIFT, PK_SMALL, PK_COUNT      // PK_SMALL also covers the column means of the centred variant
};

// Brackets one kernel launch with a HIP event pair when profiling is on.
struct ProfScope {
  rsvd_ctx *ctx; hipStream_t s; hipEvent_t stop; bool active;
  ProfScope(rsvd_ctx *c, hipStream_t st, int kind) : ctx(c), s(st), stop(nullptr), active(false) {
    if (c == nullptr || !c->prof_on) return;
    if (c->prof_used * 2 + 2 > c->prof_events.size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
      c->prof_events.push_back(a); c->prof_events.push_back(b); c->prof_kinds.push_back(kind);
    }
    c->prof_kinds[c->prof_used] = kind;
    (void)hipEventRecord(c->prof_events[c->prof_used * 2], st);
    stop = c->prof_events[c->prof_used * 2 + 1];
    c->prof_used += 1;
    active = true;
  }
  ~ProfScope() { if (active) (void)hipEventRecord(stop, s); }
};

// Device-side diagnostics block (4 x int32), same field order as rsvd_info.
struct DevInfo {
  int status;
  int jacobi_sweeps;
  int refilled;
  int skipped_reorth;
  int raised;
};
constexpr int kDevInfoInts = 5;

// ---------------------------------------------------------------- GEMM
// C (M x N) = alpha * op(A) (M x K) * B (K x N) + beta * C, row-major.
//   trans_a == 0: A is M x K (lda >= K).   trans_a != 0: A is K x M (lda >= M).
//   trans_c != 0: the result is stored transposed (C is N x M, ldc >= M); beta must be 0.
//   dead != NULL: for every column j with dead[j] != 0 the stored value is replaced by
//     refill_scale * N(0,1) drawn from Philox stream `refill_stream`, element
//     index row * refill_ld + j (used by the orthonormalisation to replace
//     linearly dependent columns).
struct GemmDesc {
  int trans_a = 0;
  int trans_c = 0;
  int64_t M = 0, N = 0, K = 0;
  const void *A = nullptr; int64_t lda = 0;
  const void *B = nullptr; int64_t ldb = 0;
  void *C = nullptr;       int64_t ldc = 0;
  double alpha = 1.0, beta = 0.0;
  // a_shift != NULL: the product is taken with A - 1 a_shift^T (one fp64 offset per column of the
  // stored A, i.e. K of them for trans_a == 0 and M for trans_a != 0), subtracted element by element
  // in fp64 while the tiles of A are staged.  Plain product only: alpha = 1, beta = 0, no trans_c,
  // no dead columns, batch = 1.
  const double *a_shift = nullptr;
  // upper_only != 0: the result is symmetric (M == N) and only its tiles on or above the diagonal
  // are computed; what lies in the tiles strictly below (and their split-K partials) is undefined.
  // Every 16 x 16 block on the diagonal is complete.
  int upper_only = 0;
  // b_upper != 0: B (K x N, K == N) is upper triangular with exact zeros below its diagonal; the k range of a
  // column tile stops where its columns of B do (the terms left out are zeros: the result is the same, bit for bit,
  // for finite A).
  int b_upper = 0;
  const int *dead = nullptr;
  uint64_t seed = 0; uint32_t refill_stream = 0; double refill_scale = 1.0; int64_t refill_ld = 0;
  void *partial = nullptr; size_t partial_bytes = 0;   // split-K scratch
  int force_splits = 0;                                 // 0 = heuristic
  int prof_kind = PK_SMALL;                             // class of the main kernel; the split-K reduction is +1
  // skip_reduce: leave split-K partials ([splits][M][N], accumulator type) unreduced in
  // `partial` for the consumer to add up; *splits_out receives their number (1 = C was written).
  int skip_reduce = 0;
  int skip_reduce_max = 1 << 30;                        // ... only when there are at most this many partials
  int *splits_out = nullptr;
  // Batched launch: `batch` equal-shaped problems, one per blockIdx.y; the pointers above are
  // those of problem 0 and problem b adds b times the matching stride (in BYTES; 0 = shared).
  int batch = 1;
  int64_t stride_a = 0, stride_b = 0, stride_c = 0, stride_partial = 0, stride_dead = 0;
  uint64_t seed_step = 0;               // problem b draws replacement columns with seed + b * seed_step
  // Device-side switches (ints in device memory, one per problem, stride_flag bytes apart):
  //   skip_flag != NULL and *skip_flag != 0: the launch (and its split-K reduction) does nothing;
  //   alt_flag != NULL and *alt_flag != 0: B_alt (same shape, leading dimension and stride as B) replaces B.
  const int *skip_flag = nullptr; const int *alt_flag = nullptr; const void *B_alt = nullptr; int64_t stride_flag = 0;
};

enum GemmKind { GEMM_F32 = 0, GEMM_F64 = 1, GEMM_F32_ACC64 = 2 };  // last: fp32 inputs, fp64 MFMA and output

// Bytes of split-K scratch the heuristic would use for this shape.
size_t gemm_partial_bytes(const rsvd_ctx *ctx, GemmKind kind, int trans_a, int64_t M, int64_t N, int64_t K);
hipError_t gemm_launch(rsvd_ctx *ctx, hipStream_t s, GemmKind kind, const GemmDesc &d);

// ---------------------------------------------------------------- sketch
// batch > 1: problem b (blockIdx.y) writes to out + b * stride_out bytes with seed + b.
hipError_t sketch_launch(hipStream_t s, rsvd_dtype dtype, uint64_t seed, uint32_t stream_id,
                         int64_t rows, int64_t cols, void *out, int64_t ld, int batch = 1, int64_t stride_out = 0);
hipError_t philox_raw_launch(hipStream_t s, uint64_t seed, uint32_t stream_id, uint64_t first_group,
                             int64_t n_groups, uint32_t *out);

// ---------------------------------------------------------------- small dense kernels
// Largest block order the single-workgroup Cholesky kernel can hold in LDS.
int chol_max_block(const rsvd_ctx *ctx);
// Upper Cholesky factor G = R^T R of the symmetric positive semi-definite fp64
// matrix G (l x l, ld ldg; overwritten), R^-1 written in `out_dtype`, and one
// flag per column that was found dependent (pivot <= tau * original diagonal).
//   Rinv (l x l, ld l, out_dtype, upper triangular, zero below)
//   R    (l x l, ld l, fp64, upper triangular, zero below) or NULL
//   dead (l ints), info->refilled += number of flagged columns
//   scratch: fp64 scratch of at least chol_scratch_elems(l) elements (blocked path)
size_t chol_scratch_elems(const rsvd_ctx *ctx, int64_t l);
//   G may be given as n_parts matrices part_stride elements apart whose sum is the
//   Gram matrix (unreduced split-K partials; single-block orders only).
//   batch > 1 (single-block orders only): problem b = blockIdx.x adds b * stride bytes to G, Rinv, R,
//   dead and info (stride 0 for info: one shared block).
//   skip_flag (device, may be NULL; strided like the rest in a batch): non-zero = do nothing.
//   pv: what happens to a pivot at or below tau * (original squared norm of its column):
//     raise = 0: the column is dropped (flagged in `dead`; the caller replaces it);
//     raise = 1: the column is set aside - it stays in Q, scaled by 1 / sqrt(threshold) instead of normalised,
//       and is not used to eliminate the later ones (only a column whose original squared norm is zero or
//       below floor_abs is dropped);
//     floor_abs: columns whose original squared norm is below this are dropped outright;
//     abs_thr > 0: the threshold is this value for every column instead of tau * (its squared norm);
//     redo_skip (device int, strided by `stride` in a batch, may be NULL): set to 0 when a pivot was raised,
//       to 1 otherwise (also when skip_flag switches the factorisation off) - the skip flag of the
//       additional CholeskyQR round that raised pivots call for.
struct CholPivoting {
  int raise = 0;
  double floor_abs = 0.0;
  double abs_thr = 0.0;
  int *redo_skip = nullptr;
};
hipError_t chol_inverse_launch(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype out_dtype, int64_t l,
                               double *G, int64_t ldg, int n_parts, int64_t part_stride, double tau,
                               void *Rinv, double *R, int *dead, DevInfo *info, double *scratch,
                               int batch = 1, int64_t stride = 0, const int *skip_flag = nullptr,
                               const CholPivoting &pv = CholPivoting());
// Once per context, with its device current: raises the dynamic-LDS limit of the kernels that need it.
hipError_t chol_init_device(rsvd_ctx *ctx);
hipError_t jacobi_init_device(rsvd_ctx *ctx);
// *flag = 1 when the Frobenius condition number ||R||_F ||R^-1||_F (an upper bound of the 2-norm one) of the
// l x l factor is at most `limit` and finite, else 0.  R fp64, Rinv in `dtype`, both l x l with ld l.
// info (may be NULL): skipped_reorth is raised to the flag.
// redo_skip (may be NULL; strided like the rest): when it reads 0 - the factorisation raised a pivot - the flag is 0.
hipError_t cond_flag_launch(hipStream_t s, rsvd_dtype dtype, int64_t l, const double *R, const void *Rinv,
                            double limit, int *flag, DevInfo *info, int batch = 1, int64_t stride = 0,
                            const int *redo_skip = nullptr);
// Rb = R2 * R1 for upper triangular fp64 l x l matrices (ld l).
hipError_t triu_product_launch(hipStream_t s, int64_t l, const double *R2, const double *R1, double *Rb,
                               int batch = 1, int64_t stride = 0, const int *skip_flag = nullptr);
hipError_t zero_ints_launch(hipStream_t s, int *p, int n, int batch = 1, int64_t stride = 0);

// ---------------------------------------------------------------- Jacobi
// Largest order the single-workgroup LDS-resident Jacobi kernel handles.
int jacobi_max_lds_order(const rsvd_ctx *ctx, rsvd_dtype dtype);
// Largest order rsvd_run_batched takes (fp64: 128, with the rotations accumulated in global memory beyond 96).
int jacobi_max_batched_order(const rsvd_ctx *ctx, rsvd_dtype dtype);
size_t jacobi_scratch_bytes(const rsvd_ctx *ctx, rsvd_dtype dtype, int64_t l);
// G = Y^T Y in fp64 for panels of at most gram_syrk_max_order() columns (Y rows x l, ld ldy, of type dtype; G l x l,
// ld l): the 16 x 16 blocks on or above the diagonal only.  The row ranges of the workgroups leave partial matrices
// ([parts][l][l] in `partial`); up to max_parts of them are left for the consumer to add (*parts_out tells how
// many; 1 = Gout holds the sum), more are added here.
int gram_syrk_max_order();
size_t gram_syrk_partial_bytes(const rsvd_ctx *ctx, int64_t rows, int64_t l);
hipError_t gram_init_device(rsvd_ctx *ctx);
hipError_t gram_syrk_launch(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype dtype, int64_t rows, int64_t l, const void *Y,
                            int64_t ldy, double *Gout, void *partial, size_t partial_bytes, int max_parts,
                            int *parts_out, int batch, int64_t stride, const int *skip_flag);

// Q = Y R^-1 for panels of at most apply_tri_max_order(dtype) columns (Y rows x l, ld ldy; R^-1 l x l upper
// triangular, ld l; Q may be Y): R^-1 resident in LDS, workgroups walking over 64-row tiles.  Columns flagged in
// `dead` are replaced by Gaussian directions (element (row, col) from counter row * refill_ld + col of Philox stream
// refill_stream, times refill_scale).  batch problems `stride` bytes apart (every pointer and the flag);
// *skip_flag != 0: nothing is done.
int apply_tri_max_order(rsvd_dtype dtype);
hipError_t apply_init_device(rsvd_ctx *ctx);
hipError_t apply_tri_launch(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype dtype, int64_t rows, int64_t l, const void *Y,
                            int64_t ldy, const void *Rinv, void *Q, int64_t ldq, const int *dead, uint64_t seed,
                            uint32_t refill_stream, double refill_scale, int64_t refill_ld, int batch, int64_t stride,
                            const int *skip_flag);

// One-sided Jacobi SVD  M = X diag(sigma) W^T  of the l x l row-major matrix M
// (ld l; fp64 when m_is_f64 else `dtype`).  Outputs in `dtype`, sigma descending.
// batch > 1 (LDS-resident orders only): problem b = blockIdx.x adds b * stride bytes to M, sigma, X, W.
// rows != 0: the rotations act on the rows of M, i.e. M^T = X diag(sigma) W^T is what is decomposed (the
// caller swaps X and W to get the factors of M).  One-sided Jacobi converges much faster on vectors of graded
// length; of a triangular factor those are the rows.
hipError_t jacobi_launch(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype dtype, int64_t l,
                         const void *M, int m_is_f64, void *sigma, void *X, void *W,
                         DevInfo *info, void *scratch, size_t scratch_bytes, int batch = 1, int64_t stride = 0,
                         int rows = 0);

}  // namespace rsvd
