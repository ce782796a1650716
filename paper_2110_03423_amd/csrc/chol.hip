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

// 1 / sqrt(d) for d > 0: hardware estimate refined by two Newton steps (error below
// 2 ulp); the pivot chain is the serial bottleneck, so it must be short.
__device__ __forceinline__ double fast_rsqrt(double d) {
  double y = __builtin_amdgcn_rsq(d);
  y = y * (1.5 - 0.5 * d * y * y);
  y = y * (1.5 - 0.5 * d * y * y);
  return y;
}

// One workgroup of TG x TG threads factors an nb x nb block (nb <= TG * NR) that
// it holds in registers: thread (ty, tx) owns the elements (ty + TG a, tx + TG b)
// of the symmetric matrix S and of Z = R^-T.  The block is the sum of n_parts
// matrices spaced part_stride elements apart (split-K partial Gram matrices are
// added here, in a fixed order).
// Right-looking elimination, one step per column j: the owners of row j publish
// it through double-buffered LDS lines (one barrier per step); every thread then
// applies the update to its elements of S (blocks on or above the block diagonal,
// whole 16 x 16 blocks so the inner loop carries no masks) and of Z.  Row j of R and column j of R^-1 are final at
// step j and go straight to global memory.
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
  __shared__ double bufS[2][LMAX], bufS1[2][LMAX];    // rows j and j+1 of S, double buffered
  __shared__ double bufZ[2][LMAX], bufZ1[2][LMAX];    // the same rows of Z
  __shared__ double d0[LMAX];
  __shared__ double zdiag[LMAX];
  __shared__ int n_dead, n_dead2, bad;
  extern __shared__ double outm[];       // nb x (LMAX + 1): finished rows of R and Z
  constexpr int ost = LMAX + 1;
  const int tid = threadIdx.x;
  const int tx = tid % TG, ty = tid / TG;
  double S[NR][NR], Z[NR][NR];

  if (tid == 0) { n_dead = 0; n_dead2 = 0; bad = 0; }
#pragma unroll
  for (int a = 0; a < NR; ++a)
#pragma unroll
    for (int b = 0; b < NR; ++b) { S[a][b] = 0.0; Z[a][b] = 0.0; }
  // all loads of a batch of parts are issued before they are added, so the memory
  // latency is paid once per batch and not once per element
  constexpr int UB = NR > 4 ? 1 : (NR > 2 ? 2 : 4);
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
      if (i == c && i == nb) { S[a][b] = 1.0; d0[i] = 1.0; }      // padding column of an odd order
    }

  // Two columns per step (a 2 x 2 pivot block): half as many barriers and LDS round
  // trips as column-by-column elimination, same arithmetic.  The loop is unrolled over
  // the 16-wide row blocks (A0 is a compile-time constant inside), so the registers that
  // hold rows j, j+1 are addressed statically and blocks that can no longer change are
  // dropped at compile time: branches inside a step cost more than the arithmetic they
  // would save.  An odd order is padded with a unit diagonal entry.
#pragma unroll
  for (int A0 = 0; A0 < NR; ++A0) {
    for (int jj = 0; jj < TG; jj += 2) {
      const int j = A0 * TG + jj;
      if (j >= nb) break;
      const int par = (j >> 1) & 1;
      double *bs0 = bufS[par], *bz0 = bufZ[par], *bs1 = bufS1[par], *bz1 = bufZ1[par];
      if (ty == jj) {
#pragma unroll
        for (int b = 0; b < NR; ++b) { bs0[tx + TG * b] = S[A0][b]; bz0[tx + TG * b] = Z[A0][b]; }
      }
      if (ty == jj + 1) {
#pragma unroll
        for (int b = 0; b < NR; ++b) { bs1[tx + TG * b] = S[A0][b]; bz1[tx + TG * b] = Z[A0][b]; }
      }
      __syncthreads();
      const double d00 = bs0[j], d01 = bs0[j + 1], d11 = bs1[j + 1];
      const double dj0 = d0[j], dj1 = d0[j + 1];
      const bool dead0 = !(d00 > tau * dj0) || !(dj0 > 0.0);
      const double rinv0 = dead0 ? 0.0 : fast_rsqrt(d00);
      const double r01 = d01 * rinv0;
      const double d11p = d11 - r01 * r01;
      const bool dead1 = !(d11p > tau * dj1) || !(dj1 > 0.0);
      const double rinv1 = dead1 ? 0.0 : fast_rsqrt(d11p);
      double s0[NR], s1[NR], z0[NR], z1[NR], l0[NR], l1[NR];
#pragma unroll
      for (int b = 0; b < NR; ++b) {
        const int c = tx + TG * b;
        const double t0 = (b >= A0) ? bs0[c] * rinv0 : 0.0;                    // R[j][c] for c > j
        s0[b] = (c > j) ? t0 : 0.0;
        s1[b] = (b >= A0 && c > j + 1) ? (bs1[c] - r01 * t0) * rinv1 : 0.0;    // R[j+1][c]
        const double u0 = (b <= A0) ? ((c < j) ? bz0[c] * rinv0 : ((c == j) ? rinv0 : 0.0)) : 0.0;   // Z[j][c]
        z0[b] = u0;
        z1[b] = (b <= A0) ? ((c <= j) ? (bz1[c] - r01 * u0) * rinv1 : ((c == j + 1) ? rinv1 : 0.0)) : 0.0;
      }
#pragma unroll
      for (int a = 0; a < NR; ++a) {
        const int i = ty + TG * a;
        const bool below = (a >= A0) && (i > j + 1);
        const double t0 = below ? bs0[i] * rinv0 : 0.0;                        // R[j][i]
        l0[a] = t0;
        l1[a] = below ? (bs1[i] - r01 * t0) * rinv1 : 0.0;                     // R[j+1][i]
      }
#pragma unroll
      for (int a = A0; a < NR; ++a)
#pragma unroll
        for (int b = 0; b < NR; ++b) {
          if (b >= a) S[a][b] = fma(-l1[a], s1[b], fma(-l0[a], s0[b], S[a][b]));   // upper block triangle only
          if (b <= A0) Z[a][b] = fma(-l1[a], z1[b], fma(-l0[a], z0[b], Z[a][b]));
        }
      // rows j, j+1 of R and of Z (= columns of R^-1) are final: park them in LDS
      if (ty == jj) {
        const double r00 = dead0 ? 0.0 : d00 * rinv0;
#pragma unroll
        for (int b = 0; b < NR; ++b) {
          const int c = tx + TG * b;
          outm[j * ost + c] = (c > j) ? s0[b] : ((c == j) ? r00 : z0[b]);
        }
        if (tx == jj) {
          zdiag[j] = rinv0;
          dead[j] = dead0 ? 1 : 0;
          if (dead0) n_dead += 1;                                  // single writer
        }
      }
      if (ty == jj + 1) {
        const double r11 = dead1 ? 0.0 : d11p * rinv1;
#pragma unroll
        for (int b = 0; b < NR; ++b) {
          const int c = tx + TG * b;
          outm[(j + 1) * ost + c] = (c > j + 1) ? s1[b] : ((c == j + 1) ? r11 : z1[b]);
        }
        if (tx == jj + 1 && j + 1 < nb) {
          zdiag[j + 1] = rinv1;
          dead[j + 1] = dead1 ? 1 : 0;
          if (dead1) n_dead2 += 1;                                 // single writer
        }
      }
    }
  }
  __syncthreads();
  // outm: upper triangle = R, strict lower triangle = Z (row i holds Z[i][:i]), zdiag = diagonal of Z
  for (int idx = tid; idx < nb * nb; idx += TG * TG) {
    const int r = idx / nb, c = idx - r * nb;
    double rr = 0.0, ri = 0.0;
    if (r < c)       { rr = outm[r * ost + c]; ri = outm[c * ost + r]; }
    else if (r == c) { rr = outm[r * ost + r]; ri = zdiag[r]; }
    if (R != nullptr) R[(int64_t)r * ldr + c] = rr;
    Rinv[(int64_t)r * ldri + c] = (TOut)ri;
  }
  __syncthreads();
  if (tid == 0 && info != nullptr) {
    if (n_dead + n_dead2 > 0) atomicAdd(&info->refilled, n_dead + n_dead2);
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
  return 128;      // 16 x 16 threads, up to 8 x 8 elements each
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
  // 256 threads (one wavefront per SIMD) keep the per-step barrier cheap; each thread
  // holds NR x NR elements of S and of Z, NR = ceil(nb / 16); above 96 the register
  // budget asks for 1024 threads with 4 x 4 elements.
  const size_t lds = (size_t)(nb + 1) * ((size_t)((nb + 15) / 16 > 6 ? 128 : ((nb + 15) / 16) * 16) + 1) * sizeof(double);
#define RSVD_CHOL_CASE(TGV, NRV)                                                                                    \
  do {                                                                                                              \
    static bool attr_set = false;                                                                                   \
    if (!attr_set) {                                                                                                \
      (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&chol_block_kernel<TOut, TGV, NRV>),                 \
                                hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);                            \
      (void)hipGetLastError();                                                                                      \
      attr_set = true;                                                                                              \
    }                                                                                                               \
    hipLaunchKernelGGL((chol_block_kernel<TOut, TGV, NRV>), dim3(1), dim3(TGV * TGV), lds, s, G, ldg, n_parts,      \
                       part_stride, nb, g0, tau, Rinv, ldri, R, ldr, dead, info);                                   \
  } while (0)
  switch ((nb + 15) / 16) {
    case 1: RSVD_CHOL_CASE(16, 1); break;
    case 2: RSVD_CHOL_CASE(16, 2); break;
    case 3: RSVD_CHOL_CASE(16, 3); break;
    case 4: RSVD_CHOL_CASE(16, 4); break;
    case 5: RSVD_CHOL_CASE(16, 5); break;
    case 6: RSVD_CHOL_CASE(16, 6); break;
    default: RSVD_CHOL_CASE(32, 4); break;
  }
#undef RSVD_CHOL_CASE
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
