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

namespace rsvd {

hipError_t gemm_launch_f64(rsvd_ctx *ctx, hipStream_t s, const GemmDesc &d);

// One workgroup of TG x TG threads factors an nb x nb block (nb <= TG * NR) that
// it holds in registers: thread (ty, tx) owns the elements (ty + TG a, tx + TG b).
// The block is the sum of n_parts matrices spaced part_stride elements apart
// (split-K partial Gram matrices are added here, in a fixed order).
// Right-looking elimination, one step per column j: the owners of row j publish
// it through a double-buffered LDS line (one barrier per step), every thread then
// updates its own elements.  The same pass carries Z = R^-T along: rows of Z live
// in the strict lower triangle, its diagonal 1 / R[j][j] in dinv.
//   g0    : original squared column norms for the pivot test, or NULL to use the diagonal
//   Rinv  : nb x nb block of R^-1 (ld ldri, type TOut, zeros below the diagonal)
//   R     : same for R in fp64 (ld ldr), or NULL
//   dead  : nb flags (1 = pivot <= tau * original squared norm)
template <typename TOut, int TG, int NR>
__global__ __launch_bounds__(TG * TG) void chol_block_kernel(const double *__restrict__ G, int64_t ldg,
                                                              int n_parts, int64_t part_stride, int nb,
                                                              const double *__restrict__ g0, double tau,
                                                              TOut *__restrict__ Rinv, int64_t ldri,
                                                              double *__restrict__ R, int64_t ldr,
                                                              int *__restrict__ dead, DevInfo *info) {
  constexpr int LMAX = TG * NR;
  __shared__ double rowbuf[2][LMAX];
  __shared__ double dinv[LMAX];
  __shared__ double d0[LMAX];
  __shared__ int n_dead, bad;
  const int tid = threadIdx.x;
  const int tx = tid % TG, ty = tid / TG;
  double S[NR][NR];

  if (tid == 0) { n_dead = 0; bad = 0; }
#pragma unroll
  for (int a = 0; a < NR; ++a)
#pragma unroll
    for (int b = 0; b < NR; ++b) S[a][b] = 0.0;
  // all NR*NR loads of a group of four parts are issued before they are added, so the
  // memory latency is paid once per group and not once per element
  constexpr int UB = (TG * TG > 256 && NR > 3) ? 2 : 4;   // parts per batch, bounded by the register budget
  for (int s0 = 0; s0 < n_parts; s0 += UB) {
    double v[UB][NR][NR];
#pragma unroll
    for (int u = 0; u < UB; ++u)
#pragma unroll
      for (int a = 0; a < NR; ++a)
#pragma unroll
        for (int b = 0; b < NR; ++b) {
          const int i = ty + TG * a, c = tx + TG * b;
          v[u][a][b] = (s0 + u < n_parts && i < nb && c < nb)
                           ? G[(int64_t)(s0 + u) * part_stride + (int64_t)i * ldg + c] : 0.0;
        }
#pragma unroll
    for (int u = 0; u < UB; ++u)
#pragma unroll
      for (int a = 0; a < NR; ++a)
#pragma unroll
        for (int b = 0; b < NR; ++b) S[a][b] += v[u][a][b];
  }
  __syncthreads();                       // n_dead / bad initialised
#pragma unroll
  for (int a = 0; a < NR; ++a)
#pragma unroll
    for (int b = 0; b < NR; ++b) {
      const int i = ty + TG * a, c = tx + TG * b;
      if (i == c && i < nb) {
        const double d = (g0 != nullptr) ? g0[i] : S[a][b];
        d0[i] = d;
        if (!(fabs(d) <= 1.79e308)) bad = 1;      // NaN or Inf
      }
    }

  for (int j = 0; j < nb; ++j) {
    double *buf = rowbuf[j & 1];
#pragma unroll
    for (int a = 0; a < NR; ++a)
      if (ty + TG * a == j) {
#pragma unroll
        for (int b = 0; b < NR; ++b) {
          const int c = tx + TG * b;
          if (c < nb) buf[c] = S[a][b];
        }
      }
    __syncthreads();
    const double d = buf[j], dj0 = d0[j];
    const bool is_dead = !(d > tau * dj0) || !(dj0 > 0.0);
    const double rjj = is_dead ? 0.0 : sqrt(d);
    const double rinv = is_dead ? 0.0 : 1.0 / rjj;
    double rowc[NR], rowi[NR];
#pragma unroll
    for (int b = 0; b < NR; ++b) {
      const int c = tx + TG * b;
      rowc[b] = (c < nb) ? buf[c] * rinv : 0.0;
    }
#pragma unroll
    for (int a = 0; a < NR; ++a) {
      const int i = ty + TG * a;
      rowi[a] = (i < nb) ? buf[i] * rinv : 0.0;
    }
#pragma unroll
    for (int a = 0; a < NR; ++a) {
      const int i = ty + TG * a;
      if (i == j) {
#pragma unroll
        for (int b = 0; b < NR; ++b) {
          const int c = tx + TG * b;
          if (c == j) {
            S[a][b] = rjj;
            dinv[j] = rinv;
            dead[j] = is_dead ? 1 : 0;
            if (is_dead) n_dead += 1;            // single writer per step
          } else {
            S[a][b] = rowc[b];
          }
        }
      } else if (i > j) {
        const double lij = rowi[a];
#pragma unroll
        for (int b = 0; b < NR; ++b) {
          const int c = tx + TG * b;
          if (c == j)                S[a][b] = -lij * rinv;
          else if (c < j || c >= i)  S[a][b] -= lij * rowc[b];
        }
      }
    }
  }
  __syncthreads();

#pragma unroll
  for (int a = 0; a < NR; ++a)
#pragma unroll
    for (int b = 0; b < NR; ++b) {
      const int i = ty + TG * a, c = tx + TG * b;
      if (i < nb && c < nb) {
        if (i < c) {
          if (R != nullptr) R[(int64_t)i * ldr + c] = S[a][b];
          Rinv[(int64_t)c * ldri + i] = (TOut)0;
        } else if (i > c) {
          if (R != nullptr) R[(int64_t)i * ldr + c] = 0.0;
          Rinv[(int64_t)c * ldri + i] = (TOut)S[a][b];
        } else {
          if (R != nullptr) R[(int64_t)i * ldr + i] = S[a][b];
          Rinv[(int64_t)i * ldri + i] = (TOut)dinv[i];
        }
      }
    }
  if (tid == 0 && info != nullptr) {
    if (n_dead > 0) atomicAdd(&info->refilled, n_dead);
    if (bad) atomicMax(&info->status, (int)RSVD_ERR_NONFINITE);
  }
}

__global__ void save_diag_kernel(const double *__restrict__ G, int64_t ldg, int l, double *__restrict__ g0) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < l) g0[j] = G[(int64_t)j * ldg + j];
}

template <typename TOut>
__global__ void convert_matrix_kernel(const double *__restrict__ src, int64_t n_elems, TOut *__restrict__ dst) {
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n_elems;
       e += (int64_t)gridDim.x * blockDim.x)
    dst[e] = (TOut)src[e];
}

__global__ void fill_zero_f64_kernel(double *__restrict__ p, int64_t n) {
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x)
    p[e] = 0.0;
}

__global__ void triu_product_kernel(int l, const double *__restrict__ R2, const double *__restrict__ R1,
                                    double *__restrict__ Rb) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (int64_t)l * l) return;
  const int i = (int)(e / l), j = (int)(e - (int64_t)i * l);
  double acc = 0.0;
  for (int t = i; t <= j; ++t) acc += R2[(int64_t)i * l + t] * R1[(int64_t)t * l + j];
  Rb[e] = acc;
}

__global__ void zero_ints_kernel(int *p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

int chol_max_block(const rsvd_ctx *ctx) {
  (void)ctx;
  return 128;      // 32 x 32 threads, 4 x 4 elements each
}

size_t chol_scratch_elems(const rsvd_ctx *ctx, int64_t l) {
  if (l <= chol_max_block(ctx)) return 0;
  // blocked path: g0 (l, padded to even) + fp64 R^-1 (l*l) + R (l*l) + product scratch (l*l)
  return (size_t)l + 1 + 3 * (size_t)l * (size_t)l;
}

template <typename TOut>
static hipError_t launch_block(hipStream_t s, const double *G, int64_t ldg, int n_parts, int64_t part_stride, int nb,
                               const double *g0, double tau, TOut *Rinv, int64_t ldri, double *R, int64_t ldr,
                               int *dead, DevInfo *info) {
  if (nb <= 32) {
    hipLaunchKernelGGL((chol_block_kernel<TOut, 16, 2>), dim3(1), dim3(256), 0, s, G, ldg, n_parts, part_stride, nb,
                       g0, tau, Rinv, ldri, R, ldr, dead, info);
  } else if (nb <= 64) {
    hipLaunchKernelGGL((chol_block_kernel<TOut, 16, 4>), dim3(1), dim3(256), 0, s, G, ldg, n_parts, part_stride, nb,
                       g0, tau, Rinv, ldri, R, ldr, dead, info);
  } else if (nb <= 96) {
    hipLaunchKernelGGL((chol_block_kernel<TOut, 32, 3>), dim3(1), dim3(1024), 0, s, G, ldg, n_parts, part_stride, nb,
                       g0, tau, Rinv, ldri, R, ldr, dead, info);
  } else {
    hipLaunchKernelGGL((chol_block_kernel<TOut, 32, 4>), dim3(1), dim3(1024), 0, s, G, ldg, n_parts, part_stride, nb,
                       g0, tau, Rinv, ldri, R, ldr, dead, info);
  }
  return hipGetLastError();
}

hipError_t chol_inverse_launch(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype out_dtype, int64_t l, double *G,
                               int64_t ldg, int n_parts, int64_t part_stride, double tau, void *Rinv, double *R,
                               int *dead, DevInfo *info, double *scratch) {
  const int nbmax = chol_max_block(ctx);
  if (l <= nbmax) {
    ProfScope ps(ctx, s, PK_CHOL);
    if (out_dtype == RSVD_F32)
      return launch_block<float>(s, G, ldg, n_parts, part_stride, (int)l, nullptr, tau, (float *)Rinv, l, R, l, dead,
                                 info);
    return launch_block<double>(s, G, ldg, n_parts, part_stride, (int)l, nullptr, tau, (double *)Rinv, l, R, l, dead,
                                info);
  }
  if (n_parts != 1) return hipErrorInvalidValue;     // the blocked path wants the reduced matrix

  // Blocked right-looking factorisation; diagonal blocks by the kernel above,
  // panels and trailing updates by the fp64 GEMM.  Rf/Xf hold R and R^-1 in fp64.
  const int nb = 96 <= nbmax ? 96 : nbmax;
  double *g0 = scratch;
  double *Xf = g0 + ((l + 1) & ~(int64_t)1);
  double *Rf = Xf + l * l;
  double *T = Rf + l * l;
  hipError_t e;
  hipLaunchKernelGGL(save_diag_kernel, dim3((unsigned)ceil_div(l, 256)), dim3(256), 0, s, G, ldg, (int)l, g0);
  hipLaunchKernelGGL(fill_zero_f64_kernel, dim3(1024), dim3(256), 0, s, Xf, 2 * l * l);
  if ((e = hipGetLastError()) != hipSuccess) return e;

  for (int64_t j0 = 0; j0 < l; j0 += nb) {
    const int64_t b = (l - j0 < nb) ? (l - j0) : nb;
    const int64_t rest = l - j0 - b;
    // diagonal block: R_jj and X_jj = R_jj^-1
    {
      ProfScope ps(ctx, s, PK_CHOL);
      e = launch_block<double>(s, G + j0 * ldg + j0, ldg, 1, 0, (int)b, g0 + j0, tau, Xf + j0 * l + j0, l,
                               Rf + j0 * l + j0, l, dead + j0, info);
    }
    if (e != hipSuccess) return e;
    if (rest > 0) {
      // panel: R[j, rest] = X_jj^T G[j, rest]
      GemmDesc p;
      p.trans_a = 1; p.M = b; p.N = rest; p.K = b;
      p.A = Xf + j0 * l + j0; p.lda = l;
      p.B = G + j0 * ldg + j0 + b; p.ldb = ldg;
      p.C = Rf + j0 * l + j0 + b; p.ldc = l;
      p.force_splits = 1;
      if ((e = gemm_launch_f64(ctx, s, p)) != hipSuccess) return e;
      // trailing update: G[rest, rest] -= R[j, rest]^T R[j, rest]
      GemmDesc t;
      t.trans_a = 1; t.M = rest; t.N = rest; t.K = b;
      t.A = Rf + j0 * l + j0 + b; t.lda = l;
      t.B = Rf + j0 * l + j0 + b; t.ldb = l;
      t.C = G + (j0 + b) * ldg + j0 + b; t.ldc = ldg;
      t.alpha = -1.0; t.beta = 1.0; t.force_splits = 1;
      if ((e = gemm_launch_f64(ctx, s, t)) != hipSuccess) return e;
    }
    if (j0 > 0) {
      // inverse, block column j: X[0:j0, j] = -X[0:j0, 0:j0] (R[0:j0, j] X_jj)
      GemmDesc a;
      a.M = j0; a.N = b; a.K = b;
      a.A = Rf + j0; a.lda = l;
      a.B = Xf + j0 * l + j0; a.ldb = l;
      a.C = T; a.ldc = b; a.force_splits = 1;
      if ((e = gemm_launch_f64(ctx, s, a)) != hipSuccess) return e;
      GemmDesc c;
      c.M = j0; c.N = b; c.K = j0;
      c.A = Xf; c.lda = l;
      c.B = T; c.ldb = b;
      c.C = Xf + j0; c.ldc = l; c.alpha = -1.0; c.force_splits = 1;
      if ((e = gemm_launch_f64(ctx, s, c)) != hipSuccess) return e;
    }
  }
  if (out_dtype == RSVD_F32) {
    hipLaunchKernelGGL((convert_matrix_kernel<float>), dim3(512), dim3(256), 0, s, Xf, l * l, (float *)Rinv);
  } else {
    hipLaunchKernelGGL((convert_matrix_kernel<double>), dim3(512), dim3(256), 0, s, Xf, l * l, (double *)Rinv);
  }
  if (R != nullptr)
    hipLaunchKernelGGL((convert_matrix_kernel<double>), dim3(512), dim3(256), 0, s, Rf, l * l, R);
  return hipGetLastError();
}

hipError_t triu_product_launch(hipStream_t s, int64_t l, const double *R2, const double *R1, double *Rb) {
  hipLaunchKernelGGL(triu_product_kernel, dim3((unsigned)ceil_div(l * l, 256)), dim3(256), 0, s, (int)l, R2, R1, Rb);
  return hipGetLastError();
}

hipError_t zero_ints_launch(hipStream_t s, int *p, int n) {
  hipLaunchKernelGGL(zero_ints_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, s, p, n);
  return hipGetLastError();
}

}  // namespace rsvd
