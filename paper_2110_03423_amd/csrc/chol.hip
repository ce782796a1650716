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

hipError_t gemm_launch_f64(const rsvd_ctx *ctx, hipStream_t s, const GemmDesc &d);

constexpr int kCholThreads = 1024;

// One workgroup factors the nb x nb block at G (leading dimension ldg) held in LDS.
// S (stride nb+1): on exit the upper triangle holds R, the strict lower triangle
// holds Z = R^-T (row i, columns < i) and dinv[i] = Z[i][i] = 1 / R[i][i].
//   g0    : original squared column norms for the pivot test, or NULL to use diag(G)
//   Rinv  : nb x nb block of R^-1 written at Rinv (ld ldri), type TOut, full block
//           (zeros below the diagonal)
//   R     : same for R in fp64 (ld ldr), or NULL
//   dead  : nb flags
template <typename TOut>
__global__ __launch_bounds__(kCholThreads) void chol_block_kernel(const double *__restrict__ G, int64_t ldg,
                                                                  int nb, const double *__restrict__ g0,
                                                                  double tau, TOut *__restrict__ Rinv,
                                                                  int64_t ldri, double *__restrict__ R,
                                                                  int64_t ldr, int *__restrict__ dead,
                                                                  DevInfo *info) {
  extern __shared__ double lds[];
  const int st = nb + 1;
  double *S = lds;                 // nb * st
  double *dinv = S + nb * st;      // nb
  double *d0 = dinv + nb;          // nb
  __shared__ int n_dead, bad;
  const int tid = threadIdx.x, nt = blockDim.x;
  const int tx = tid & 63, ty = tid >> 6, nwave = nt >> 6;

  if (tid == 0) { n_dead = 0; bad = 0; }
  for (int idx = tid; idx < nb * nb; idx += nt) {
    const int r = idx / nb, c = idx - r * nb;
    S[r * st + c] = G[(int64_t)r * ldg + c];
  }
  __syncthreads();
  for (int j = tid; j < nb; j += nt) {
    const double d = (g0 != nullptr) ? g0[j] : S[j * st + j];
    d0[j] = d;
    if (!(fabs(d) <= 1.79e308)) bad = 1;      // NaN or Inf
  }
  __syncthreads();

  for (int j = 0; j < nb; ++j) {
    const double d = S[j * st + j];
    const bool is_dead = !(d > tau * d0[j]) || !(d0[j] > 0.0);
    const double rjj = is_dead ? 0.0 : sqrt(d);
    const double rinv = is_dead ? 0.0 : 1.0 / rjj;
    __syncthreads();                       // everyone has read the pivot
    // scale row j: R[j][j+1:] and Z[j][:j]
    for (int c = tid; c < nb; c += nt) {
      if (c == j) {
        S[j * st + j] = rjj;
        dinv[j] = rinv;
        dead[j] = is_dead ? 1 : 0;
        if (is_dead) n_dead += 1;          // single writer per step
      } else {
        S[j * st + c] *= rinv;
      }
    }
    __syncthreads();
    // rank-one update of the rows below: trailing part of G and rows of Z
    for (int i = j + 1 + ty; i < nb; i += nwave) {
      const double lij = S[j * st + i];
      if (lij != 0.0) {
        for (int c = tx; c < nb; c += 64) {
          if (c < j)        S[i * st + c] -= lij * S[j * st + c];
          else if (c == j)  S[i * st + c] = -lij * dinv[j];
          else if (c >= i)  S[i * st + c] -= lij * S[j * st + c];
        }
      } else if (tx == 0) {
        S[i * st + j] = 0.0;
      }
    }
    // next iteration starts with a barrier after the pivot read; one more here so
    // the pivot read sees the finished update
    __syncthreads();
  }

  for (int idx = tid; idx < nb * nb; idx += nt) {
    const int r = idx / nb, c = idx - r * nb;
    double ri = 0.0, rr = 0.0;
    if (r < c)       { ri = S[c * st + r]; rr = S[r * st + c]; }
    else if (r == c) { ri = dinv[r];       rr = S[r * st + r]; }
    Rinv[(int64_t)r * ldri + c] = (TOut)ri;
    if (R != nullptr) R[(int64_t)r * ldr + c] = rr;
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
  // nb * (nb + 1) + 2 nb doubles of dynamic LDS, plus a little static
  int nb = 128;
  while (nb > 16 && ((size_t)nb * (nb + 1) + 2 * (size_t)nb) * 8 + 256 > ctx->lds_per_block) nb -= 16;
  return nb;
}

size_t chol_scratch_elems(const rsvd_ctx *ctx, int64_t l) {
  if (l <= chol_max_block(ctx)) return 0;
  // blocked path: g0 (l) + fp64 R^-1 (l*l) + R (l*l) + product scratch (l*l)
  return (size_t)l + 3 * (size_t)l * (size_t)l;
}

template <typename TOut>
static hipError_t launch_block(hipStream_t s, const double *G, int64_t ldg, int nb, const double *g0, double tau,
                               TOut *Rinv, int64_t ldri, double *R, int64_t ldr, int *dead, DevInfo *info) {
  const size_t lds = ((size_t)nb * (nb + 1) + 2 * (size_t)nb) * sizeof(double);
  const int threads = nb <= 32 ? 256 : (nb <= 64 ? 512 : kCholThreads);
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&chol_block_kernel<TOut>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 512);
    (void)hipGetLastError();
    attr_set = true;
  }
  hipLaunchKernelGGL((chol_block_kernel<TOut>), dim3(1), dim3(threads), lds, s, G, ldg, nb, g0, tau, Rinv, ldri, R,
                     ldr, dead, info);
  return hipGetLastError();
}

hipError_t chol_inverse_launch(const rsvd_ctx *ctx, hipStream_t s, rsvd_dtype out_dtype, int64_t l, double *G,
                               int64_t ldg, double tau, void *Rinv, double *R, int *dead, DevInfo *info,
                               double *scratch, void *partial, size_t partial_bytes) {
  const int nbmax = chol_max_block(ctx);
  if (l <= nbmax) {
    if (out_dtype == RSVD_F32)
      return launch_block<float>(s, G, ldg, (int)l, nullptr, tau, (float *)Rinv, l, R, l, dead, info);
    return launch_block<double>(s, G, ldg, (int)l, nullptr, tau, (double *)Rinv, l, R, l, dead, info);
  }

  // Blocked right-looking factorisation; diagonal blocks by the kernel above,
  // panels and trailing updates by the fp64 GEMM.  Rf/Xf hold R and R^-1 in fp64.
  const int nb = 96 <= nbmax ? 96 : nbmax;
  double *g0 = scratch;
  double *Xf = g0 + l;
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
    e = launch_block<double>(s, G + j0 * ldg + j0, ldg, (int)b, g0 + j0, tau, Xf + j0 * l + j0, l,
                             Rf + j0 * l + j0, l, dead + j0, info);
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
  (void)partial; (void)partial_bytes;
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
