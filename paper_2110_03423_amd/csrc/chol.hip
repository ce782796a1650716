// Step 3 of Algorithm 1, small dense part: the l x l work of CholeskyQR.
//
// The paper orthonormalises the tall-skinny Y with Householder QR
// (GEQRF + ORGQR).  Here the same Q (up to column signs) comes from the Gram
// matrix: G = Y^T Y = R^T R, Q = Y R^-1, applied twice.  This file factors G
// and inverts R in fp64.  A pivot that drops below tau times the column's
// original squared norm marks the column as numerically dependent: its row of
// R and its column of R^-1 are set to zero (the caller replaces the column of
// Q by a fresh Gaussian direction), so a rank-deficient Y still gives a full
// orthonormal basis that contains range(Y).
#include "common.hpp"
#include "mfma.hpp"

namespace rsvd {

hipError_t gemm_launch_f64(rsvd_ctx *ctx, hipStream_t s, const GemmDesc &d);

// 1 / sqrt(d) for d > 0: hardware estimate refined by two Newton steps (error below
// 2 ulp); the pivot chain is the serial bottleneck, so it must be short.
__device__ __forceinline__ double fast_rsqrt(double d) {
  double y = __builtin_amdgcn_rsq(d);
  y = y * (1.5 - 0.5 * d * y * y);
  y = y * (1.5 - 0.5 * d * y * y);
  return y;
}

// 64-bit lane read (the lane index is a compile-time constant where this is used).
__device__ __forceinline__ double readlane_f64(double v, int lane) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
  return __hiloint2double(hi, lo);
}

// One workgroup of NB wavefronts factors an nb x nb block (nb <= 16 NB) and inverts the
// factor.  The block is the sum of n_parts matrices spaced part_stride elements apart
// (split-K partial Gram matrices are added here, in a fixed order).
//
// Elimination on [S | I] by 16 x 16 blocks.  Wavefront r owns block row r for the whole
// run and keeps it in registers in the accumulator layout of the fp64 matrix-core
// instruction: slot J >= r is the S block (r, J), slot J < r the block (r, J) of
// Z = R^-T.  Wavefront 0, whose own row is complete after the first step, factors all the
// diagonal blocks (diag_factor).  The chain that every
// step has to wait for is: row kb complete -> update of the next diagonal block -> its
// factorisation -> scaling of row kb + 1 by T^T, T = R_kk^-1; everything else is moved off it.
// Step kb, two barriers:
//   * row kb lies in LDS unscaled, T and R_kk are there: every other wavefront multiplies one
//     column block of the row by T^T on the matrix cores, in place (one block each instead of the
//     whole row in one wavefront); wavefront kb + 1, which has just scaled the block above its own
//     diagonal block, updates that block with it and hands it over through LDS;        -- barrier
//   * wavefront 0 factors block kb + 1 and publishes R, T and the flags, while the
//     wavefronts r > kb take  block(r, J) -= R[kb][r]^T block(kb, J)  for their (other) slots,
//     wavefront kb + 1 then leaves its row in LDS; behind that every wavefront but the factoring
//     one writes its share of block row kb of R and block column kb of R^-1 (the transpose
//     of Z).                                                                           -- barrier
//   g0    : original squared column norms for the pivot test, or NULL to use the diagonal
//   Rinv  : nb x nb block of R^-1 (ld ldri, type TOut, zeros below the diagonal)
//   R     : same for R in fp64 (ld ldr), or NULL
//   dead  : nb flags (1 = pivot <= tau * original squared norm)
template <int NB> struct CholLds {
  static constexpr int LP = 16 * NB, LD = LP + 1, TLD = 17;
  // rows of [R | Z], the inverses of the diagonal blocks, the reference norms, the diagonal block in hand
  static constexpr size_t bytes = ((size_t)LP * LD + (size_t)NB * 16 * TLD + LP + 256) * sizeof(double);
};

// Factor and invert one 16 x 16 symmetric block held in the accumulator layout
// (register v of lane L: row 4 v + L / 16, column L % 16).  One wavefront runs this
// alone and a lone wavefront issues about one instruction every five cycles, so the cost
// is the number of instructions per column; everything is arranged to keep that small.
// Square-root-free elimination: column j is eliminated by ONE matrix-core instruction per
// block, a rank-one update whose operands are row j itself (it already sits in the lanes
// that feed k-slot j % 4), once for the block and once for the identity next to it.  The
// update is not masked: rows that are already finished are copied out first (sd, sz) and
// what the update leaves in their place is never read.  Rows are scaled by 1 / sqrt(d_j)
// at the end.
//   dblk : in  S_kk, out R_kk (valid on and above the diagonal)
//   z    : out Z_kk = R_kk^-T (lower triangular)
//   thr  : lane c holds tau * (reference squared norm of column c); pos: bit c set when that norm is > 0
//          (and not below the caller's absolute floor)
//   piv  : 16 doubles of LDS scratch
//   raise: a pivot at or below its threshold (with a usable reference norm) does not drop its column but SETS IT
//          ASIDE: the pivot takes the value of the threshold, the row is not used to eliminate anything (its
//          part of R is the diagonal element alone), so the column comes out of Q = Y R^-1 as what is left of it
//          after the columns before it, divided by sqrt(threshold): short of unit length, with the direction it
//          still carries magnified to where the next round can resolve it, and with no large entries in R^-1
//          (eliminating with a raised pivot instead couples the weak rows by ratios far above one, and their
//          inverse overflowed on a sketch with ~100 such rows)
//   returns the 16-bit mask of dropped (dependent) columns, and in bits 16..31 that of the columns set aside
__device__ __forceinline__ unsigned diag_factor(f64x4 &dblk, f64x4 &z, double thr, unsigned pos, int lane,
                                                double *piv, bool raise) {
  const int lr = lane >> 4, lc = lane & 15;
  double mrow[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) mrow[q] = (lr == q) ? 1.0 : 0.0;
#pragma unroll
  for (int v = 0; v < 4; ++v) z[v] = (4 * v + lr == lc) ? 1.0 : 0.0;
  f64x4 sd = {0.0, 0.0, 0.0, 0.0}, sz = {0.0, 0.0, 0.0, 0.0};
  unsigned dmask = 0, wmask = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int q = j & 3, v4 = j >> 2;
    double rowv = dblk[v4];
    const double d = readlane_f64(rowv, 16 * q + j);            // pivot S[j][j]
    const unsigned gt = (unsigned)__ballot(d > thr);            // bit c: d exceeds the threshold of column c
    double y = __builtin_amdgcn_rcp(d);
    y = fma(fma(-d, y, 1.0), y, y);        // the hardware estimate is good to ~1e-8: one step squares that
    if (!(((gt & pos) >> j) & 1u)) {                            // pivot at the rounding level of the Gram matrix (rare)
      y = 0.0;                                                  // no elimination with this row
      if (raise && ((pos >> j) & 1u)) {
        const double dr = readlane_f64(thr, j);                 // lane j holds the threshold of column j
        wmask |= 1u << j;
        if (lane == 16 * q + j) rowv = dr;                      // the diagonal element of the row takes the raised value
      } else {
        dmask |= 1u << j;                                       // dependent column
      }
    }
    const double b_d = rowv * mrow[q];
    const double b_z = z[v4] * mrow[q];
    const double a_op = b_d * -y;
    sd[v4] += b_d;
    sz[v4] += b_z;
    dblk = Mfma<double>::run(a_op, b_d, dblk);
    z = Mfma<double>::run(a_op, b_z, z);
  }
  // pivot of row i = diagonal element of the saved row: pass it along the lane row through LDS
#pragma unroll
  for (int v = 0; v < 4; ++v)
    if (lc == 4 * v + lr) piv[lc] = sd[v];
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const double x = piv[4 * v + lr];
    double rv = __builtin_amdgcn_rsq(x);
    rv = rv * (1.5 - 0.5 * x * rv * rv);
    rv = rv * (1.5 - 0.5 * x * rv * rv);
    if ((dmask >> (4 * v + lr)) & 1u) rv = 0.0;
    dblk[v] = sd[v] * rv;
    if (((wmask >> (4 * v + lr)) & 1u) && lc != 4 * v + lr) dblk[v] = 0.0;      // set aside: the diagonal alone
    z[v] = sz[v] * rv;
  }
  return dmask | (wmask << 16);
}

template <typename TOut, int NB>
__global__ __launch_bounds__(NB * 64) void chol_mfma_kernel(const double *__restrict__ G, int64_t ldg,
                                                                  int n_parts, int64_t part_stride, int nb,
                                                                  const double *__restrict__ g0, double tau,
                                                                  TOut *__restrict__ Rinv, int64_t ldri,
                                                                  double *__restrict__ R, int64_t ldr,
                                                                  int *__restrict__ dead, DevInfo *info,
                                                                  int64_t stride, const int *skip_flag, int raise,
                                                                  double floor_abs, double abs_thr, int *redo_skip,
                                                                  int redo_mode, double *__restrict__ Rinv_elim,
                                                                  int64_t ldre) {
  typedef CholLds<NB> L;
  // redo_skip (device int, strided like the rest in a batch; may be NULL): the switch of the additional
  // CholeskyQR round that follows a factorisation with raised pivots; non-zero = that round is skipped.
  //   redo_mode 1: this launch decides alone: 0 when it raised a pivot, 1 when not (and when it is skipped itself);
  //   redo_mode 2: one of several launches of a blocked factorisation: only ever clears it.
  // Rinv_elim (fp64, ld ldre, may be NULL): a second copy of R^-1 whose columns of set-aside rows are zero.  A blocked
  // factorisation forms its panel R[j, rest] = X_jj^T G[j, rest] with it, so that the rows set aside come out zero
  // there as they do inside this kernel, and take no part in the trailing update.
  if (redo_skip != nullptr)
    redo_skip = reinterpret_cast<int *>(reinterpret_cast<char *>(redo_skip) + (int64_t)blockIdx.x * stride);
  if (skip_flag != nullptr &&
      *reinterpret_cast<const int *>(reinterpret_cast<const char *>(skip_flag) + (int64_t)blockIdx.x * stride) != 0) {
    if (redo_skip != nullptr && redo_mode == 1 && threadIdx.x == 0) *redo_skip = 1;
    return;
  }
  if (blockIdx.x != 0) {              // batched launch: one problem per workgroup, `stride` bytes apart
    const int64_t off = (int64_t)blockIdx.x * stride;
    G = reinterpret_cast<const double *>(reinterpret_cast<const char *>(G) + off);
    Rinv = reinterpret_cast<TOut *>(reinterpret_cast<char *>(Rinv) + off);
    if (R != nullptr) R = reinterpret_cast<double *>(reinterpret_cast<char *>(R) + off);
    dead = reinterpret_cast<int *>(reinterpret_cast<char *>(dead) + off);
  }
  constexpr int LP = L::LP, LD = L::LD, TLD = L::TLD;
  extern __shared__ double smem[];
  double *Sm = smem;                       // LP x LD: rows of [R | Z]
  double *Td = Sm + LP * LD;               // NB x 16 x TLD: R_kk^-1
  double *d0 = Td + NB * 16 * TLD;         // LP: reference squared norms for the pivot test
  double *Dg = d0 + LP;                    // 4 x 64: the diagonal block in hand, accumulator layout
  __shared__ double piv[16];
  __shared__ int n_dead, n_weak, bad;
  __shared__ unsigned wmask_sh;            // rows of the current pivot block that were set aside
  __shared__ unsigned char aside[16 * NB];
  const int tid = threadIdx.x, lane = tid & 63;
  // Block row of this wavefront; the wavefront of row 0 also factors the diagonal blocks.  Wavefronts w and w + 4
  // share a SIMD unit and its matrix pipe: the one next to the factoring wavefront takes row 1, which is complete
  // after the first step, so that the factorisations that follow have the pipe to themselves.
  const int wv = tid >> 6;
  const int wr = NB > 4 ? (wv == 4 ? 1 : (wv == 1 ? 4 : wv)) : wv;
  const int lr = lane >> 4, lc = lane & 15;
  // register slot t of wavefront wr holds column block (wr + t) mod NB: slot 0 is the
  // diagonal block, slots 1 .. NB-1-wr the S blocks to its right, the rest the Z blocks
  auto col_block = [&](int t) { const int J = wr + t; return J >= NB ? J - NB : J; };

  if (tid == 0) { n_dead = 0; n_weak = 0; bad = 0; wmask_sh = 0u; }
  __syncthreads();
  // ---- load block row wr: sum of the parts for the S slots, zero for the Z slots, identity padding
  f64x4 acc[NB];
#pragma unroll
  for (int t = 0; t < NB; ++t) acc[t] = f64x4{0.0, 0.0, 0.0, 0.0};
  {
    const double *Gr = G + (int64_t)(16 * wr + lr) * ldg + 16 * wr + lc;
    for (int p = 0; p < n_parts; ++p) {
      f64x4 cur[NB];
#pragma unroll
      for (int t = 0; t < NB; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int row = 16 * wr + 4 * v + lr, col = 16 * (wr + t) + lc;
          cur[t][v] = (row < nb && col < nb) ? Gr[(int64_t)p * part_stride + (int64_t)(4 * v) * ldg + 16 * t] : 0.0;
        }
#pragma unroll
      for (int t = 0; t < NB; ++t) acc[t] += cur[t];
    }
    // reference norms of this row's 16 columns; unit diagonal in the padding
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = 16 * wr + 4 * v + lr;
      if (4 * v + lr != lc) continue;          // the lane that holds the diagonal element of this row
      double dv = 1.0;
      if (row < nb) dv = (g0 != nullptr) ? g0[row] : acc[0][v];
      else acc[0][v] = 1.0;
      d0[row] = dv;
      if (!(fabs(dv) <= 1.79e308)) bad = 1;      // NaN or Inf
    }
  }

  // Wavefront 0: factor the block in Dg as diagonal block kb, publish R_kk, T = R_kk^-1 and the flags.
  auto factor_block = [&](int kb) {
    const int k0 = kb * 16;
    f64x4 dblk, z;
#pragma unroll
    for (int v = 0; v < 4; ++v) dblk[v] = Dg[v * 64 + lane];
    const double d0c = d0[k0 + lc];
    const unsigned pos = (unsigned)__ballot(d0c > 0.0 && d0c >= floor_abs) & 0xffffu;
    // pivot threshold: tau times the column's reference norm, or the same for every column (abs_thr > 0:
    // rounds that work on a panel whose resolved columns have unit length)
    const unsigned masks = diag_factor(dblk, z, abs_thr > 0.0 ? abs_thr : tau * d0c, pos, lane, piv, raise != 0);
    const unsigned dmask = masks & 0xffffu, wmask = masks >> 16;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = 4 * v + lr;
      Sm[(k0 + row) * LD + k0 + lc] = (lc >= row) ? dblk[v] : 0.0;          // R_kk
      Td[(k0 + lc) * TLD + row] = z[v];                                      // T[c][row] = Z[row][c]
    }
    if (lane < 16 && k0 + lane < nb) dead[k0 + lane] = (int)((dmask >> lane) & 1u);
    if (lane < 16) aside[k0 + lane] = (unsigned char)((wmask >> lane) & 1u);
    if (lane == 0) {
      const int valid = min(16, nb - k0);
      n_dead += __popc(dmask & ((1u << valid) - 1u));     // wavefront 0 is the only writer
      n_weak += __popc(wmask & ((1u << valid) - 1u));
      wmask_sh = wmask;
    }
  };
  // Row wavefront wr leaves its diagonal block in Dg and the rest of its row, unscaled, in LDS.
  auto put_diag = [&]() {
#pragma unroll
    for (int v = 0; v < 4; ++v) Dg[v * 64 + lane] = acc[0][v];
  };
  auto put_row = [&]() {
#pragma unroll
    for (int t = 1; t < NB; ++t) {
      double *dst = Sm + (16 * wr + lr) * LD + 16 * col_block(t) + lc;
#pragma unroll
      for (int v = 0; v < 4; ++v) dst[4 * v * LD] = acc[t][v];
    }
  };

  if (wr == 0) { put_diag(); put_row(); }
  __syncthreads();
  if (wr == 0) factor_block(0);
  __syncthreads();

#pragma unroll 1
  for (int kb = 0; kb < NB; ++kb) {
    const int k0 = kb * 16;
    // ---- row kb times T^T, in place: wavefront J takes column block J (R to the right of the diagonal, Z to the left)
    if (wr != kb) {
      double ta[4], bo[4];
      double *blk = Sm + (k0 + lr) * LD + 16 * wr + lc;
#pragma unroll
      for (int s = 0; s < 4; ++s) { ta[s] = Td[(k0 + 4 * s + lr) * TLD + lc]; bo[s] = blk[4 * s * LD]; }
      f64x4 o = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int s = 0; s < 4; ++s) o = Mfma<double>::run(ta[s], bo[s], o);
      const unsigned wmask = wmask_sh;
      if (wr > kb && wmask != 0u) {
        // rows set aside keep nothing of R to the right of the diagonal (their part of R^-1, the Z blocks, stays)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if ((wmask >> (4 * v + lr)) & 1u) o[v] = 0.0;
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) blk[4 * v * LD] = o[v];
      if (wr == kb + 1) {
        // the next pivot row brings its diagonal block up to date with the block it has just scaled (the
        // accumulator layout is the layout of both operands:  block(wr, wr) -= R[kb][wr]^T R[kb][wr])
        // and hands it over
#pragma unroll
        for (int s = 0; s < 4; ++s) acc[0] = Mfma<double>::run(-o[s], o[s], acc[0]);
        put_diag();
      }
    }
    __syncthreads();
    if (wr > kb) {
      // ---- trailing rows: block(wr, J) -= R[kb][wr]^T block(kb, J)
      double na[4], b[NB][4];
#pragma unroll
      for (int s = 0; s < 4; ++s) na[s] = -Sm[(k0 + 4 * s + lr) * LD + 16 * wr + lc];
#pragma unroll
      for (int t = 0; t < NB; ++t) {
        const int J = col_block(t);
        const bool on = !(J > kb && J < wr);       // an S slot (J >= wr) or a touched Z slot (J <= kb)
        const double *src = (J == kb) ? Td + (k0 + lc) * TLD + lr                   // Z_kk = T_kk^T
                                      : Sm + (k0 + lr) * LD + 16 * J + lc;
        const int step = (J == kb) ? 4 : 4 * LD;
#pragma unroll
        for (int s = 0; s < 4; ++s) b[t][s] = on ? src[s * step] : 0.0;      // untouched slots take a zero update
      }
      // (slot loop innermost: consecutive matrix-core instructions are independent)
      if (wr == kb + 1) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
          for (int t = 1; t < NB; ++t) acc[t] = Mfma<double>::run(na[s], b[t][s], acc[t]);
        put_row();
      } else {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
          for (int t = 0; t < NB; ++t) acc[t] = Mfma<double>::run(na[s], b[t][s], acc[t]);
      }
    } else if (wr == 0 && kb + 1 < NB) {
      factor_block(kb + 1);
    }
    // ---- block row kb of R and block column kb of R^-1 are written out (R^-1 = Z^T: column k0 + c of R^-1 is
    // row k0 + c of Z) by every wavefront but the one that factors, each behind its update: off the critical path
    const bool last = kb + 1 == NB;
    if (wr != 0 || last) {
      const int parts = NB - 1 + (last ? 1 : 0), me = wr == 0 ? NB - 1 : wr - 1;
      const int ldr_i = (int)ldr, ldri_i = (int)ldri;      // orders here are at most a few hundred
      if (R != nullptr) {
        const int rows = min(16, nb - k0);
        for (int c = lane; c < nb; c += 64) {
#pragma unroll 4
          for (int i = me; i < rows; i += parts) {
            const int r = k0 + i;
            R[r * ldr_i + c] = (c >= r) ? Sm[r * LD + c] : 0.0;
          }
        }
      }
      const int c = k0 + lc;
      if (c < nb) {
#pragma unroll 4
        for (int r = lr + 4 * me; r < nb; r += 4 * parts) {
          double v = 0.0;
          if (r <= c) v = (r >= k0) ? Td[r * TLD + lc] : Sm[c * LD + r];
          Rinv[r * ldri_i + c] = (TOut)v;
          if (Rinv_elim != nullptr) Rinv_elim[r * (int)ldre + c] = aside[c] ? 0.0 : v;
        }
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    if (info != nullptr) {
      if (n_dead > 0) atomicAdd(&info->refilled, n_dead);
      if (n_weak > 0) atomicAdd(&info->raised, n_weak);
      if (bad) atomicMax(&info->status, (int)RSVD_ERR_NONFINITE);
    }
    if (redo_skip != nullptr) {
      if (redo_mode == 1) *redo_skip = (n_weak > 0) ? 0 : 1;
      else if (n_weak > 0) *redo_skip = 0;
    }
  }
}

// First launch of a blocked factorisation: keeps the original diagonal for the pivot tests and arms the switch
// of the additional round (see chol_mfma_kernel) - also when the factorisation itself is switched off.
__global__ void save_diag_kernel(const double *__restrict__ G, int64_t ldg, int l, double *__restrict__ g0,
                                 const int *skip_flag, int *redo_skip) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j == 0 && redo_skip != nullptr) *redo_skip = 1;
  if (skip_flag != nullptr && *skip_flag != 0) return;
  if (j < l) g0[j] = G[(int64_t)j * ldg + j];
}

template <typename TOut>
__global__ void convert_matrix_kernel(const double *__restrict__ src, int64_t n_elems, TOut *__restrict__ dst,
                                      const int *skip_flag) {
  if (skip_flag != nullptr && *skip_flag != 0) return;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_elems;
       e += (int64_t)gridDim.x * blockDim.x)
    dst[e] = (TOut)src[e];
}

__global__ void fill_zero_f64_kernel(double *__restrict__ p, int64_t n, const int *skip_flag) {
  if (skip_flag != nullptr && *skip_flag != 0) return;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x)
    p[e] = 0.0;
}

__global__ void triu_product_kernel(int l, const double *__restrict__ R2, const double *__restrict__ R1,
                                    double *__restrict__ Rb, int64_t stride, const int *skip_flag) {
  const int64_t off = (int64_t)blockIdx.y * stride;        // batched: bytes between problems
  if (skip_flag != nullptr && *reinterpret_cast<const int *>(reinterpret_cast<const char *>(skip_flag) + off) != 0)
    return;
  R2 = reinterpret_cast<const double *>(reinterpret_cast<const char *>(R2) + off);
  R1 = reinterpret_cast<const double *>(reinterpret_cast<const char *>(R1) + off);
  Rb = reinterpret_cast<double *>(reinterpret_cast<char *>(Rb) + off);
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (int64_t)l * l) return;
  const int i = (int)(e / l), j = (int)(e - (int64_t)i * l);
  // eight products per step with all their loads issued first (one at a time, every term would wait
  // for its own memory round trip)
  double acc = 0.0;
  for (int t0 = i; t0 <= j; t0 += 8) {
    double a[8], b[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int t = t0 + u;
      a[u] = (t <= j) ? R2[(int64_t)i * l + t] : 0.0;
      b[u] = (t <= j) ? R1[(int64_t)t * l + j] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc = fma(a[u], b[u], acc);
  }
  Rb[e] = acc;
}

__global__ void zero_ints_kernel(int *p, int n, int64_t stride) {
  p = reinterpret_cast<int *>(reinterpret_cast<char *>(p) + (int64_t)blockIdx.y * stride);
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

int chol_max_block(const rsvd_ctx *ctx) {
  (void)ctx;
  return 128;      // 8 x 8 blocks of 16 x 16 in 149 KB of LDS
}

size_t chol_scratch_elems(const rsvd_ctx *ctx, int64_t l) {
  if (l <= chol_max_block(ctx)) return 0;
  // blocked path: g0 (l, padded to even) + fp64 R^-1 (l*l) + R (l*l) + product scratch (l*l) + the inverse of one
  // diagonal block with the columns of set-aside rows cleared (128 x 128)
  return (size_t)l + 1 + 3 * (size_t)l * (size_t)l + 128 * 128;
}

template <typename TOut>
static hipError_t launch_block(hipStream_t s, const double *G, int64_t ldg, int n_parts, int64_t part_stride, int nb,
                               const double *g0, double tau, TOut *Rinv, int64_t ldri, double *R, int64_t ldr,
                               int *dead, DevInfo *info, int batch, int64_t stride, const int *skip_flag,
                               const CholPivoting &pv, int redo_mode, double *Rinv_elim = nullptr,
                               int64_t ldre = 0) {
  // one workgroup, one wavefront per 16-row block
#define RSVD_CHOL_CASE(NBV)                                                                                         \
  hipLaunchKernelGGL((chol_mfma_kernel<TOut, NBV>), dim3(batch), dim3(NBV * 64), CholLds<NBV>::bytes, s, G,         \
                     ldg, n_parts, part_stride, nb, g0, tau, Rinv, ldri, R, ldr, dead, info, stride, skip_flag,     \
                     pv.raise, pv.floor_abs, pv.abs_thr, pv.redo_skip, redo_mode, Rinv_elim, ldre)
  switch ((nb + 15) / 16) {
    case 1: RSVD_CHOL_CASE(1); break;
    case 2: RSVD_CHOL_CASE(2); break;
    case 3: RSVD_CHOL_CASE(3); break;
    case 4: RSVD_CHOL_CASE(4); break;
    case 5: RSVD_CHOL_CASE(5); break;
    case 6: RSVD_CHOL_CASE(6); break;
    case 7: RSVD_CHOL_CASE(7); break;
    case 8: RSVD_CHOL_CASE(8); break;
    default: return hipErrorInvalidValue;
  }
#undef RSVD_CHOL_CASE
  return hipGetLastError();
}

// The kernels of this file that need more LDS than the default limit of a launch: raised once per context.
template <typename TOut>
static hipError_t chol_raise_lds_limits() {
  hipError_t e = hipSuccess;
#define RSVD_CHOL_ATTR(NBV)                                                                              \
  if (e == hipSuccess)                                                                                   \
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&chol_mfma_kernel<TOut, NBV>),                \
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)CholLds<NBV>::bytes)
  RSVD_CHOL_ATTR(1); RSVD_CHOL_ATTR(2); RSVD_CHOL_ATTR(3); RSVD_CHOL_ATTR(4);
  RSVD_CHOL_ATTR(5); RSVD_CHOL_ATTR(6); RSVD_CHOL_ATTR(7); RSVD_CHOL_ATTR(8);
#undef RSVD_CHOL_ATTR
  return e;
}

// Blocks of X = R^-1 above the diagonal blocks, given R (upper triangular, l x l) and the inverted diagonal
// blocks X_jj (nb x nb, nb = 16 * NW) already in place in X.  Column c of X depends on nothing but R and the
// X_ii: block row i of a column is  X_i = -X_ii (R[i, i+1 ..] X[i+1 .., c]),  from the diagonal block upwards.  So
// one workgroup takes a strip of 16 columns through the whole back substitution with the strip in LDS, every
// strip at once - one launch where a blocked forward scheme needs two small products per block column, each
// waiting for the one before.  Wavefront w owns rows 16 w .. 16 w + 15 of the block row in hand.
//   LDS: the strip ((rows up to the end of its diagonal block) x 17), one block row of products (nb x 17) and
//   a chunk of R (nb x 34).
template <int NW>
__global__ __launch_bounds__(64 * NW) void tri_inverse_strip_kernel(const double *__restrict__ R,
                                                                    double *__restrict__ X, int l,
                                                                    const int *skip_flag) {
  if (skip_flag != nullptr && *skip_flag != 0) return;
  constexpr int nb = 16 * NW, LDS_ = 17;
  const int c0 = (int)blockIdx.x * 16;
  const int j = c0 / nb, j0 = j * nb;
  if (j == 0) return;                                   // the first block column is its diagonal block
  const int kend = (j0 + nb < l) ? j0 + nb : l;         // rows of the strip that the diagonal block supplies end here
  extern __shared__ double tri_smem[];
  double *Xs = tri_smem;                                // [kend][17]
  double *Ts = Xs + (size_t)kend * LDS_;                // [nb][17]
  constexpr int CK = 32, RLD = CK + 2;                  // chunk of R: nb rows x CK columns, padded rows
  constexpr int PER = (nb * (CK / 2) + 64 * NW - 1) / (64 * NW);   // pairs of elements per thread and chunk
  double *Rs = Ts + (size_t)nb * LDS_;                  // [nb][RLD]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int r16 = lane & 15, kq = lane >> 4;
  for (int idx = tid; idx < (kend - j0) * 16; idx += 64 * NW) {
    const int r = j0 + idx / 16, c = idx % 16;
    Xs[r * LDS_ + c] = (c0 + c < l) ? X[(int64_t)r * l + c0 + c] : 0.0;
  }
  __syncthreads();
  for (int i = j - 1; i >= 0; --i) {
    const int i0 = i * nb;
    // operands of the second product (row 16 w + r16 of X_ii, columns 16 w ..): independent of everything this
    // kernel computes, so they travel while the first product runs
    constexpr int NX = nb / 4;
    double xv[NX];
    {
      const double *Xrow = X + (int64_t)(i0 + 16 * w + r16) * l + i0;
#pragma unroll
      for (int u = 0; u < NX; ++u) {
        const int k = 16 * w + 4 * u + kq;
        xv[u] = (k < nb) ? Xrow[k] : 0.0;
      }
    }
    // Ts = R[i0 : i0 + nb, i0 + nb : kend] Xs[i0 + nb : kend, :], the block row of R staged through LDS in
    // chunks of CK columns with coalesced loads (a lane fetching its own row of R touches sixteen cache lines
    // per instruction, and that, not the arithmetic, was the whole cost of a first version)
    {
      f64x4 acc = {0.0, 0.0, 0.0, 0.0};
      double stage[2 * PER];
      auto fetch = [&](int kk) {
#pragma unroll
        for (int t = 0; t < PER; ++t) {
          const int e = tid + 64 * NW * t;                  // pair of columns e % (CK / 2) of row e / (CK / 2)
          const int row = e / (CK / 2), k = kk + 2 * (e % (CK / 2));
          const double *src = R + (int64_t)(i0 + row) * l + k;
          stage[2 * t] = (row < nb && k < kend) ? src[0] : 0.0;
          stage[2 * t + 1] = (row < nb && k + 1 < kend) ? src[1] : 0.0;
        }
      };
      fetch(i0 + nb);
      for (int kk = i0 + nb; kk < kend; kk += CK) {
#pragma unroll
        for (int t = 0; t < PER; ++t) {
          const int e = tid + 64 * NW * t;
          const int row = e / (CK / 2), c = 2 * (e % (CK / 2));
          if (row < nb) {
            Rs[row * RLD + c] = stage[2 * t];
            Rs[row * RLD + c + 1] = stage[2 * t + 1];
          }
        }
        __syncthreads();
        if (kk + CK < kend) fetch(kk + CK);
#pragma unroll
        for (int u = 0; u < CK / 4; ++u) {
          const int k = kk + 4 * u + kq;
          const double bv = (k < kend) ? Xs[k * LDS_ + r16] : 0.0;
          acc = Mfma<double>::run(Rs[(16 * w + r16) * RLD + 4 * u + kq], bv, acc);
        }
        __syncthreads();
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) Ts[(16 * w + Mfma<double>::row(lane, v)) * LDS_ + r16] = acc[v];
    }
    __syncthreads();
    // Xs[i0 : i0 + nb, :] = -X_ii Ts   (X_ii is upper triangular: columns from this row block on; its operands
    // were fetched before the product above)
    {
      f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int u = 0; u < NX; ++u) {
        const int k = 16 * w + 4 * u + kq;
        const double bv = (k < nb) ? Ts[k * LDS_ + r16] : 0.0;
        acc = Mfma<double>::run(xv[u], bv, acc);
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) Xs[(i0 + 16 * w + Mfma<double>::row(lane, v)) * LDS_ + r16] = -acc[v];
    }
    __syncthreads();
  }
  for (int idx = tid; idx < j0 * 16; idx += 64 * NW) {
    const int r = idx / 16, c = idx % 16;
    if (c0 + c < l) X[(int64_t)r * l + c0 + c] = Xs[r * LDS_ + c];
  }
}

hipError_t chol_init_device(rsvd_ctx *ctx) {
  (void)ctx;
  hipError_t e = chol_raise_lds_limits<float>();
  if (e == hipSuccess) e = chol_raise_lds_limits<double>();
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tri_inverse_strip_kernel<6>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 4096);
  return e;
}

hipError_t chol_inverse_launch(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype out_dtype, int64_t l, double *G,
                               int64_t ldg, int n_parts, int64_t part_stride, double tau, void *Rinv, double *R,
                               int *dead, DevInfo *info, double *scratch, int batch, int64_t stride,
                               const int *skip_flag, const CholPivoting &pv) {
  const int nbmax = chol_max_block(ctx);
  if (batch < 1 || batch > 65535) return hipErrorInvalidValue;
  if (l <= nbmax) {
    ProfScope ps(ctx, s, PK_CHOL);
    if (out_dtype == RSVD_F32)
      return launch_block<float>(s, G, ldg, n_parts, part_stride, (int)l, nullptr, tau, (float *)Rinv, l, R, l, dead,
                                 info, batch, stride, skip_flag, pv, 1);
    return launch_block<double>(s, G, ldg, n_parts, part_stride, (int)l, nullptr, tau, (double *)Rinv, l, R, l, dead,
                                info, batch, stride, skip_flag, pv, 1);
  }
  if (batch != 1) return hipErrorNotSupported;       // the blocked path is not batched
  if (n_parts != 1) return hipErrorInvalidValue;     // the blocked path wants the reduced matrix

  // Blocked right-looking factorisation; diagonal blocks by the kernel above,
  // panels and trailing updates by the fp64 GEMM.  Rf/Xf hold R and R^-1 in fp64.
  const int nb = 96 <= nbmax ? 96 : nbmax;
  // R^-1 above the diagonal blocks: one strip kernel after the factorisation when its strip fits in LDS
  // (l up to ~1000), else two products per block column inside the loop
  const size_t strip_lds = ((size_t)(l + nb) * 17 + (size_t)nb * 34) * sizeof(double);
  const bool strips = nb == 96 && strip_lds + 4096 <= (size_t)ctx->lds_per_block;
  double *g0 = scratch;
  double *Xf = g0 + ((l + 1) & ~(int64_t)1);
  double *Rf = Xf + l * l;
  double *T = Rf + l * l;
  double *E = T + l * l;               // nb x nb (ld nb): X_jj without the columns of rows set aside
  const bool aside = pv.raise != 0;
  hipError_t e;
  hipLaunchKernelGGL(save_diag_kernel, dim3((unsigned)ceil_div(l, 256)), dim3(256), 0, s, G, ldg, (int)l, g0,
                     skip_flag, pv.redo_skip);
  hipLaunchKernelGGL(fill_zero_f64_kernel, dim3(1024), dim3(256), 0, s, Xf, 2 * l * l, skip_flag);
  if ((e = hipGetLastError()) != hipSuccess) return e;

  for (int64_t j0 = 0; j0 < l; j0 += nb) {
    const int64_t b = (l - j0 < nb) ? (l - j0) : nb;
    const int64_t rest = l - j0 - b;
    // diagonal block: R_jj and X_jj = R_jj^-1
    {
      ProfScope ps(ctx, s, PK_CHOL);
      e = launch_block<double>(s, G + j0 * ldg + j0, ldg, 1, 0, (int)b, g0 + j0, tau, Xf + j0 * l + j0, l,
                               Rf + j0 * l + j0, l, dead + j0, info, 1, 0, skip_flag, pv, 2, aside ? E : nullptr, nb);
    }
    if (e != hipSuccess) return e;
    if (rest > 0) {
      // panel: R[j, rest] = X_jj^T G[j, rest]
      GemmDesc p;
      p.trans_a = 1; p.M = b; p.N = rest; p.K = b;
      p.A = aside ? E : Xf + j0 * l + j0; p.lda = aside ? nb : l;
      p.B = G + j0 * ldg + j0 + b; p.ldb = ldg;
      p.C = Rf + j0 * l + j0 + b; p.ldc = l;
      p.force_splits = 1; p.skip_flag = skip_flag;
      if ((e = gemm_launch_f64(ctx, s, p)) != hipSuccess) return e;
      // trailing update: G[rest, rest] -= R[j, rest]^T R[j, rest]
      GemmDesc t;
      t.trans_a = 1; t.M = rest; t.N = rest; t.K = b;
      t.A = Rf + j0 * l + j0 + b; t.lda = l;
      t.B = Rf + j0 * l + j0 + b; t.ldb = l;
      t.C = G + (j0 + b) * ldg + j0 + b; t.ldc = ldg;
      t.alpha = -1.0; t.beta = 1.0; t.force_splits = 1;
      t.upper_only = 1;                 // nothing below reads the lower triangle of G
      t.skip_flag = skip_flag;
      if ((e = gemm_launch_f64(ctx, s, t)) != hipSuccess) return e;
    }
    if (j0 > 0 && !strips) {
      // inverse, block column j: X[0:j0, j] = -X[0:j0, 0:j0] (R[0:j0, j] X_jj)
      GemmDesc a;
      a.M = j0; a.N = b; a.K = b;
      a.A = Rf + j0; a.lda = l;
      a.B = Xf + j0 * l + j0; a.ldb = l;
      a.C = T; a.ldc = b; a.force_splits = 1; a.skip_flag = skip_flag;
      if ((e = gemm_launch_f64(ctx, s, a)) != hipSuccess) return e;
      GemmDesc c;
      c.M = j0; c.N = b; c.K = j0;
      c.A = Xf; c.lda = l;
      c.B = T; c.ldb = b;
      c.C = Xf + j0; c.ldc = l; c.alpha = -1.0; c.force_splits = 1; c.skip_flag = skip_flag;
      if ((e = gemm_launch_f64(ctx, s, c)) != hipSuccess) return e;
    }
  }
  if (strips) {
    ProfScope ps(ctx, s, PK_SMALL);
    hipLaunchKernelGGL((tri_inverse_strip_kernel<6>), dim3((unsigned)ceil_div(l, 16)), dim3(384), strip_lds, s, Rf, Xf,
                       (int)l, skip_flag);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (out_dtype == RSVD_F32) {
    hipLaunchKernelGGL((convert_matrix_kernel<float>), dim3(512), dim3(256), 0, s, Xf, l * l, (float *)Rinv, skip_flag);
  } else {
    hipLaunchKernelGGL((convert_matrix_kernel<double>), dim3(512), dim3(256), 0, s, Xf, l * l, (double *)Rinv,
                       skip_flag);
  }
  if (R != nullptr)
    hipLaunchKernelGGL((convert_matrix_kernel<double>), dim3(512), dim3(256), 0, s, Rf, l * l, R, skip_flag);
  return hipGetLastError();
}

// One workgroup per problem: sums of squares of R and of R^-1, flag = (their product <= limit^2).
template <typename T>
__global__ __launch_bounds__(1024) void cond_flag_kernel(int l, const double *__restrict__ R, const T *__restrict__ Rinv,
                                                         double limit, int *flag, DevInfo *info, int64_t stride,
                                                         const int *redo_skip) {
  const int64_t off = (int64_t)blockIdx.x * stride;
  // a factorisation with raised pivots: the panel is badly conditioned whatever the later factors look like
  const bool raised = redo_skip != nullptr &&
                      *reinterpret_cast<const int *>(reinterpret_cast<const char *>(redo_skip) + off) == 0;
  R = reinterpret_cast<const double *>(reinterpret_cast<const char *>(R) + off);
  Rinv = reinterpret_cast<const T *>(reinterpret_cast<const char *>(Rinv) + off);
  flag = reinterpret_cast<int *>(reinterpret_cast<char *>(flag) + off);
  __shared__ double part[2][16];
  __shared__ int singular;
  if (threadIdx.x == 0) singular = 0;
  __syncthreads();
  double a = 0.0, b = 0.0;
  {
    // sixteen loads in flight per thread (one after the other, l = 576 took 150 us here)
    const int nt = (int)blockDim.x, total = l * l;
    int e = threadIdx.x;
    for (; e + 7 * nt < total; e += 8 * nt) {
      double rv[8], xv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) { rv[u] = R[e + u * nt]; xv[u] = (double)Rinv[e + u * nt]; }
#pragma unroll
      for (int u = 0; u < 8; ++u) { a += rv[u] * rv[u]; b += xv[u] * xv[u]; }
    }
    for (; e < total; e += nt) {
      const double r = R[e], x = (double)Rinv[e];
      a += r * r;
      b += x * x;
    }
  }
  for (int j = threadIdx.x; j < l; j += blockDim.x)
    if (!(fabs((double)Rinv[j * l + j]) > 0.0)) singular = 1;       // a column was flagged dependent (or NaN)
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { a += __shfl_xor(a, o, 64); b += __shfl_xor(b, o, 64); }
  if ((threadIdx.x & 63) == 0) { part[0][threadIdx.x >> 6] = a; part[1][threadIdx.x >> 6] = b; }
  __syncthreads();
  if (threadIdx.x == 0) {
    a = 0.0; b = 0.0;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) { a += part[0][w]; b += part[1][w]; }
    const double k2 = a * b;                     // (||R||_F ||R^-1||_F)^2 >= cond_2(R)^2
    const int f = (!raised && !singular && k2 > 0.0 && k2 <= limit * limit) ? 1 : 0;      // NaN and Inf give 0
    *flag = f;
    if (f && info != nullptr) atomicMax(&info->skipped_reorth, 1);
  }
}

hipError_t cond_flag_launch(hipStream_t s, rsvd_dtype dtype, int64_t l, const double *R, const void *Rinv,
                            double limit, int *flag, DevInfo *info, int batch, int64_t stride, const int *redo_skip) {
  if (dtype == RSVD_F32)
    hipLaunchKernelGGL(cond_flag_kernel<float>, dim3(batch), dim3(1024), 0, s, (int)l, R, (const float *)Rinv, limit,
                       flag, info, stride, redo_skip);
  else
    hipLaunchKernelGGL(cond_flag_kernel<double>, dim3(batch), dim3(1024), 0, s, (int)l, R, (const double *)Rinv, limit,
                       flag, info, stride, redo_skip);
  return hipGetLastError();
}

hipError_t triu_product_launch(hipStream_t s, int64_t l, const double *R2, const double *R1, double *Rb, int batch,
                               int64_t stride, const int *skip_flag) {
  hipLaunchKernelGGL(triu_product_kernel, dim3((unsigned)ceil_div(l * l, 256), (unsigned)batch), dim3(256), 0, s,
                     (int)l, R2, R1, Rb, stride, skip_flag);
  return hipGetLastError();
}

hipError_t zero_ints_launch(hipStream_t s, int *p, int n, int batch, int64_t stride) {
  hipLaunchKernelGGL(zero_ints_kernel, dim3((unsigned)ceil_div(n, 256), (unsigned)batch), dim3(256), 0, s, p, n,
                     stride);
  return hipGetLastError();
}

}  // namespace rsvd
