// Step 5 of Algorithm 1: SVD of the small factor by one-sided Jacobi rotations.
//
// The paper's step 5 uses a Jacobi solver because up to n/2 disjoint plane
// rotations can run in parallel and a handful of sweeps suffice.  Here the
// l x l matrix M (the triangular factor of B^T) is held column-major in LDS by
// one workgroup; each sweep walks a round-robin tournament of l-1 rounds, and in
// every round the l/2 disjoint column pairs are rotated concurrently, one
// sub-wavefront group of lanes per pair.  Rotations are accumulated in J, so on
// convergence  M J = X diag(sigma)  and  M = X diag(sigma) J^T.
//
// Stopping rule (the paper gives none): a sweep in which every pair satisfies
// |a_p . a_q| <= tol * ||a_p|| * ||a_q||, tol = eps * sqrt(l); at most 30 sweeps.
// A column whose norm has fallen below eps * ||M||_F counts as zero and is no
// longer rotated (rotating it would change its partner by less than the
// rounding level); without this floor the surplus columns of a rank-deficient M
// keep shrinking by a factor eps per sweep until they underflow.  Its singular
// value is reported as that norm and its column of X is set to zero.
#include "common.hpp"

namespace rsvd {

constexpr int kJacobiMaxSweeps = 30;

template <typename T> struct Eps;
template <> struct Eps<float>  { static constexpr float  value = 1.1920929e-07f; };
template <> struct Eps<double> { static constexpr double value = 2.220446049250313e-16; };

// Pair i of round r in a tournament of n2 (even) players: player n2-1 stays,
// the others rotate (circle method).
__device__ __forceinline__ void tournament_pair(int n2, int r, int i, int &a, int &b) {
  const int nm1 = n2 - 1;
  if (i == 0) {
    a = nm1;
    b = r % nm1;
  } else {
    a = (r + i) % nm1;
    b = (r - i + nm1) % nm1;
  }
}

// Rotate columns p, q of M (and of J) held column-major with stride ldm; the G
// lanes of one group share the work, each holding up to RPL elements of either
// column in registers between the inner products and the update.  Returns true
// when a rotation was applied.
template <typename T, int G, int RPL>
__device__ __forceinline__ bool rotate_pair(T *Mc, T *Jc, int ldm, int rows, int p, int q, int lg, T tol,
                                            T floor2) {
  T *mp = Mc + p * ldm, *mq = Mc + q * ldm;
  T x[RPL], y[RPL];
  T alpha = 0, beta = 0, gamma = 0;
#pragma unroll
  for (int r = 0; r < RPL; ++r) {
    const int i = lg + G * r;
    const bool ok = i < rows;
    x[r] = ok ? mp[i] : (T)0;
    y[r] = ok ? mq[i] : (T)0;
  }
#pragma unroll
  for (int r = 0; r < RPL; ++r) {
    alpha += x[r] * x[r];
    beta += y[r] * y[r];
    gamma += x[r] * y[r];
  }
#pragma unroll
  for (int off = G / 2; off > 0; off >>= 1) {
    alpha += __shfl_xor(alpha, off, G);
    beta += __shfl_xor(beta, off, G);
    gamma += __shfl_xor(gamma, off, G);
  }
  if (alpha <= floor2 || beta <= floor2) return false;
  const T limit = tol * sqrt(alpha) * sqrt(beta);
  if (!(fabs(gamma) > limit)) return false;
  T *jp = Jc + p * ldm, *jq = Jc + q * ldm;
  T u[RPL], v[RPL];
#pragma unroll
  for (int r = 0; r < RPL; ++r) {
    const int i = lg + G * r;
    const bool ok = i < rows;
    u[r] = ok ? jp[i] : (T)0;
    v[r] = ok ? jq[i] : (T)0;
  }
  const T zeta = (beta - alpha) / ((T)2 * gamma);
  T t;
  if (fabs(zeta) > (T)1e7) {
    t = (T)0.5 / zeta;                         // avoids overflow of zeta^2
  } else {
    t = (zeta >= 0 ? (T)1 : (T)-1) / (fabs(zeta) + sqrt((T)1 + zeta * zeta));
  }
  const T c = (T)1 / sqrt((T)1 + t * t), s = c * t;
#pragma unroll
  for (int r = 0; r < RPL; ++r) {
    const int i = lg + G * r;
    if (i < rows) {
      mp[i] = c * x[r] - s * y[r];
      mq[i] = s * x[r] + c * y[r];
      jp[i] = c * u[r] - s * v[r];
      jq[i] = s * u[r] + c * v[r];
    }
  }
  return true;
}

template <typename T, typename TIn, int G>
__global__ __launch_bounds__(1024) void jacobi_lds_kernel(const TIn *__restrict__ M, int l, T *__restrict__ sigma,
                                                          T *__restrict__ X, T *__restrict__ W, DevInfo *info) {
  extern __shared__ double lds_raw[];
  const int ldm = l | 1;
  T *Mc = reinterpret_cast<T *>(lds_raw);
  T *Jc = Mc + (size_t)l * ldm;
  T *nrm = Jc + (size_t)l * ldm;
  int *rnk = reinterpret_cast<int *>(nrm + l);
  __shared__ int rotations;
  __shared__ T wave_sum[16];

  const int tid = threadIdx.x, nt = blockDim.x;
  T fro2 = 0;
  for (int idx = tid; idx < l * l; idx += nt) {
    const int r = idx / l, c = idx - r * l;
    const T v = (T)M[idx];
    Mc[c * ldm + r] = v;
    Jc[c * ldm + r] = (r == c) ? (T)1 : (T)0;
    fro2 += v * v;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) fro2 += __shfl_xor(fro2, off, 64);
  if ((tid & 63) == 0) wave_sum[tid >> 6] = fro2;
  if (tid == 0) rotations = 0;
  __syncthreads();
  fro2 = 0;
  for (int w = 0; w < (nt >> 6); ++w) fro2 += wave_sum[w];
  const T floor2 = Eps<T>::value * Eps<T>::value * fro2;

  const int n2 = l + (l & 1), npairs = n2 / 2;
  const int group = tid / G, lg = tid % G, ngroups = nt / G;
  const T tol = Eps<T>::value * sqrt((T)l);
  int sweeps = 0;
  bool converged = (l < 2);
  while (!converged && sweeps < kJacobiMaxSweeps) {
    ++sweeps;
    for (int r = 0; r < n2 - 1; ++r) {
      for (int pi = group; pi < npairs; pi += ngroups) {
        int a, b;
        tournament_pair(n2, r, pi, a, b);
        if (a < l && b < l) {
          const int p = a < b ? a : b, q = a < b ? b : a;
          const bool rot = rotate_pair<T, G, (128 + G - 1) / G>(Mc, Jc, ldm, l, p, q, lg, tol, floor2);
          if (rot && lg == 0) atomicAdd(&rotations, 1);
        }
      }
      __syncthreads();
    }
    converged = (rotations == 0);
    __syncthreads();
    if (tid == 0) rotations = 0;
    __syncthreads();
  }

  for (int j = tid; j < l; j += nt) {
    T s2 = 0;
    for (int i = 0; i < l; ++i) { const T x = Mc[j * ldm + i]; s2 += x * x; }
    nrm[j] = sqrt(s2);
  }
  __syncthreads();
  for (int j = tid; j < l; j += nt) {
    const T mine = nrm[j];
    int rank = 0;
    for (int i = 0; i < l; ++i) {
      const T o = nrm[i];
      rank += (o > mine || (o == mine && i < j)) ? 1 : 0;
    }
    rnk[j] = rank;
    sigma[rank] = mine;
  }
  __syncthreads();
  for (int idx = tid; idx < l * l; idx += nt) {
    const int r = idx / l, c = idx - r * l;
    const int dst = r * l + rnk[c];
    const T s = nrm[c];
    X[dst] = (s * s > floor2) ? Mc[c * ldm + r] / s : (T)0;
    W[dst] = Jc[c * ldm + r];
  }
  if (tid == 0 && info != nullptr) {
    atomicMax(&info->jacobi_sweeps, sweeps);
    if (!converged) atomicMax(&info->status, (int)RSVD_ERR_NO_CONVERGENCE);
  }
}

static size_t jacobi_lds_bytes(rsvd_dtype dtype, int64_t l) {
  const size_t es = dtype_size(dtype);
  const size_t ldm = (size_t)(l | 1);
  return align_up(2 * (size_t)l * ldm * es + (size_t)l * (es + sizeof(int)), 16);
}

int jacobi_max_lds_order(const rsvd_ctx *ctx, rsvd_dtype dtype) {
  int l = 2;
  while (l < 128 && jacobi_lds_bytes(dtype, l + 1) + 512 <= ctx->lds_per_block) ++l;
  return l;      // 128 = lanes per pair x elements each lane keeps in registers
}

size_t jacobi_scratch_bytes(const rsvd_ctx *ctx, rsvd_dtype dtype, int64_t l) {
  (void)ctx; (void)dtype; (void)l;
  return 0;
}

template <typename T, typename TIn, int G>
static hipError_t launch_lds(hipStream_t s, int nt, size_t lds, const void *M, int l, void *sigma, void *X, void *W,
                             DevInfo *info) {
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&jacobi_lds_kernel<T, TIn, G>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 512);
    (void)hipGetLastError();
    attr_set = true;
  }
  hipLaunchKernelGGL((jacobi_lds_kernel<T, TIn, G>), dim3(1), dim3(nt), lds, s, (const TIn *)M, l, (T *)sigma,
                     (T *)X, (T *)W, info);
  return hipGetLastError();
}

template <typename T, typename TIn>
static hipError_t launch_lds_g(hipStream_t s, int nt, int g, size_t lds, const void *M, int l, void *sigma, void *X,
                               void *W, DevInfo *info) {
  switch (g) {
    case 64: return launch_lds<T, TIn, 64>(s, nt, lds, M, l, sigma, X, W, info);
    case 32: return launch_lds<T, TIn, 32>(s, nt, lds, M, l, sigma, X, W, info);
    default: return launch_lds<T, TIn, 16>(s, nt, lds, M, l, sigma, X, W, info);
  }
}

hipError_t jacobi_launch(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype dtype, int64_t l, const void *M,
                         int m_is_f64, void *sigma, void *X, void *W, DevInfo *info, void *scratch,
                         size_t scratch_bytes) {
  (void)scratch; (void)scratch_bytes;
  if (l > jacobi_max_lds_order(ctx, dtype)) return hipErrorNotSupported;
  const int nt = l > 64 ? 1024 : (l > 32 ? 512 : 256);
  const int npairs = (int)((l + 1) / 2);
  int g = 64;
  while (g > 16 && nt / g < npairs) g /= 2;
  const size_t lds = jacobi_lds_bytes(dtype, l);
  ProfScope ps(ctx, s, PK_JACOBI);
  if (dtype == RSVD_F32) {
    if (m_is_f64) return launch_lds_g<float, double>(s, nt, g, lds, M, (int)l, sigma, X, W, info);
    return launch_lds_g<float, float>(s, nt, g, lds, M, (int)l, sigma, X, W, info);
  }
  return launch_lds_g<double, double>(s, nt, g, lds, M, (int)l, sigma, X, W, info);
}

}  // namespace rsvd
