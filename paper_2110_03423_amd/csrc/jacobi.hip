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

// ---------------------------------------------------------------- orders beyond one workgroup's LDS
//
// Block one-sided Jacobi.  M^T and J^T live in global memory (column c of M is
// row c of Mt, contiguous).  The columns are cut into blocks of b; an outer
// sweep is a round-robin tournament over the blocks, one kernel launch per
// round, one workgroup per block pair.  The workgroup pulls its two blocks
// (2b columns of length l) into LDS, runs inner sweeps of the same pairwise
// rotations as above over those columns while accumulating them in a small
// 2b x 2b matrix T, writes the columns back and applies T to the matching
// columns of J.  Every rotation is an exact plane rotation of actual columns of
// M, so accuracy and the stopping rule are those of the plain method.
// counters[s] collects the rotations of outer sweep s; a launch of sweep s > 0
// that finds counters[s-1] == 0 returns at once (converged), which keeps the
// whole sequence free of host synchronisation.

template <typename T, int G>
__device__ __forceinline__ bool rotate_pair_loop(T *Pc, T *Tc, int ldp, int ldt, int rows_m, int rows_t, int p,
                                                 int q, int lg, T tol, T floor2) {
  T *mp = Pc + p * ldp, *mq = Pc + q * ldp;
  T alpha = 0, beta = 0, gamma = 0;
  for (int i = lg; i < rows_m; i += G) {
    const T x = mp[i], y = mq[i];
    alpha += x * x;
    beta += y * y;
    gamma += x * y;
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
  const T zeta = (beta - alpha) / ((T)2 * gamma);
  T t;
  if (fabs(zeta) > (T)1e7) t = (T)0.5 / zeta;
  else t = (zeta >= 0 ? (T)1 : (T)-1) / (fabs(zeta) + sqrt((T)1 + zeta * zeta));
  const T c = (T)1 / sqrt((T)1 + t * t), s = c * t;
  for (int i = lg; i < rows_m; i += G) {
    const T x = mp[i], y = mq[i];
    mp[i] = c * x - s * y;
    mq[i] = s * x + c * y;
  }
  T *tp = Tc + p * ldt, *tq = Tc + q * ldt;
  for (int i = lg; i < rows_t; i += G) {
    const T x = tp[i], y = tq[i];
    tp[i] = c * x - s * y;
    tq[i] = s * x + c * y;
  }
  return true;
}

// scratch header shared by the block-Jacobi kernels
struct JbHeader {
  double fro2;            // ||M||_F^2
  int counters[64];       // rotations per outer sweep
};

template <typename T>
__global__ __launch_bounds__(1024) void jb_init_kernel(const double *__restrict__ M, int l, T *__restrict__ Mt,
                                                       T *__restrict__ Jt, JbHeader *hdr) {
  __shared__ double wave_sum[16];
  const int tid = threadIdx.x, nt = blockDim.x;
  double fro2 = 0;
  for (int64_t idx = tid; idx < (int64_t)l * l; idx += nt) {
    const int r = (int)(idx / l), c = (int)(idx - (int64_t)r * l);
    const T v = (T)M[idx];
    Mt[(int64_t)c * l + r] = v;
    Jt[idx] = (r == c) ? (T)1 : (T)0;
    fro2 += (double)v * (double)v;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) fro2 += __shfl_xor(fro2, off, 64);
  if ((tid & 63) == 0) wave_sum[tid >> 6] = fro2;
  __syncthreads();
  if (tid == 0) {
    double t = 0;
    for (int w = 0; w < (nt >> 6); ++w) t += wave_sum[w];
    hdr->fro2 = t;
  }
  if (tid < 64) hdr->counters[tid] = 0;
}

template <typename T, int G>
__global__ __launch_bounds__(1024) void jb_panel_kernel(T *__restrict__ Mt, T *__restrict__ Jt, int l, int b,
                                                        int nblk, int round, int sweep, int inner_sweeps,
                                                        JbHeader *hdr) {
  if (sweep > 0 && hdr->counters[sweep - 1] == 0) return;      // converged in the previous sweep
  const int nblk2 = nblk + (nblk & 1);
  int ba, bb;
  tournament_pair(nblk2, round, blockIdx.x, ba, bb);
  if (ba >= nblk || bb >= nblk) return;                        // bye
  const int bi = ba < bb ? ba : bb, bj = ba < bb ? bb : ba;
  const int cols_i = (l - bi * b < b) ? (l - bi * b) : b;
  const int cols_j = (l - bj * b < b) ? (l - bj * b) : b;
  const int ncols = cols_i + cols_j;

  extern __shared__ double lds_raw[];
  const int ldp = l | 1, ldt = (2 * b) | 1;
  T *Pc = reinterpret_cast<T *>(lds_raw);
  T *Tc = Pc + (size_t)(2 * b) * ldp;
  __shared__ int rotations, total;

  const int tid = threadIdx.x, nt = blockDim.x;
  auto gcol = [&](int c) { return c < cols_i ? bi * b + c : bj * b + (c - cols_i); };
  for (int c = tid / 64; c < ncols; c += nt / 64) {
    const T *src = Mt + (int64_t)gcol(c) * l;
    for (int r = tid & 63; r < l; r += 64) Pc[c * ldp + r] = src[r];
  }
  for (int idx = tid; idx < ncols * ncols; idx += nt) {
    const int c = idx / ncols, r = idx - c * ncols;
    Tc[c * ldt + r] = (r == c) ? (T)1 : (T)0;
  }
  if (tid == 0) { rotations = 0; total = 0; }
  __syncthreads();

  const T floor2 = (T)(Eps<T>::value * Eps<T>::value * hdr->fro2);
  const T tol = Eps<T>::value * sqrt((T)l);
  const int n2 = ncols + (ncols & 1), npairs = n2 / 2;
  const int group = tid / G, lg = tid % G, ngroups = nt / G;
  for (int isw = 0; isw < inner_sweeps; ++isw) {
    for (int r = 0; r < n2 - 1; ++r) {
      for (int pi = group; pi < npairs; pi += ngroups) {
        int a, c2;
        tournament_pair(n2, r, pi, a, c2);
        if (a < ncols && c2 < ncols) {
          const int p = a < c2 ? a : c2, q = a < c2 ? c2 : a;
          const bool rot = rotate_pair_loop<T, G>(Pc, Tc, ldp, ldt, l, ncols, p, q, lg, tol, floor2);
          if (rot && lg == 0) atomicAdd(&rotations, 1);
        }
      }
      __syncthreads();
    }
    const int done = rotations;
    __syncthreads();
    if (tid == 0) { total += rotations; rotations = 0; }
    __syncthreads();
    if (done == 0) break;
  }
  const int n_rot = total;
  if (n_rot == 0) return;                                     // nothing changed: leave M and J alone

  for (int c = tid / 64; c < ncols; c += nt / 64) {
    T *dst = Mt + (int64_t)gcol(c) * l;
    for (int r = tid & 63; r < l; r += 64) dst[r] = Pc[c * ldp + r];
  }
  __syncthreads();
  // J[:, panel] <- J[:, panel] T, staged through the LDS space of the panel
  for (int c = tid / 64; c < ncols; c += nt / 64) {
    const T *src = Jt + (int64_t)gcol(c) * l;
    for (int r = tid & 63; r < l; r += 64) Pc[c * ldp + r] = src[r];
  }
  __syncthreads();
  for (int r = tid; r < l; r += nt) {
    for (int cn = 0; cn < ncols; ++cn) {
      T acc = 0;
      const T *tcol = Tc + cn * ldt;                           // column cn of T: new column = sum_c T[c][cn] * old column c
      for (int c = 0; c < ncols; ++c) acc += tcol[c] * Pc[c * ldp + r];
      Jt[(int64_t)gcol(cn) * l + r] = acc;
    }
  }
  if (tid == 0) atomicAdd(&hdr->counters[sweep], n_rot);
}

// Column norms (one wavefront per column), then ranks by counting, then the scatter.
template <typename T>
__global__ __launch_bounds__(256) void jb_norms_kernel(const T *__restrict__ Mt, int l, T *__restrict__ nrm) {
  const int col = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (col >= l) return;
  T s2 = 0;
  for (int r = lane; r < l; r += 64) { const T x = Mt[(int64_t)col * l + r]; s2 += x * x; }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s2 += __shfl_xor(s2, off, 64);
  if (lane == 0) nrm[col] = sqrt(s2);
}

template <typename T>
__global__ __launch_bounds__(256) void jb_rank_kernel(const T *__restrict__ nrm, int l, int *__restrict__ rnk,
                                                      T *__restrict__ sigma, JbHeader *hdr, int max_sweeps,
                                                      DevInfo *info) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < l) {
    const T mine = nrm[j];
    int rank = 0;
    for (int i = 0; i < l; ++i) {
      const T o = nrm[i];
      rank += (o > mine || (o == mine && i < j)) ? 1 : 0;
    }
    rnk[j] = rank;
    sigma[rank] = mine;
  }
  if (j == 0 && info != nullptr) {
    int used = max_sweeps;
    for (int s = 0; s < max_sweeps; ++s)
      if (hdr->counters[s] == 0) { used = s + 1; break; }
    atomicMax(&info->jacobi_sweeps, used);
    if (hdr->counters[max_sweeps - 1] != 0) atomicMax(&info->status, (int)RSVD_ERR_NO_CONVERGENCE);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void jb_scatter_kernel(const T *__restrict__ Mt, const T *__restrict__ Jt, int l,
                                                         const T *__restrict__ nrm, const int *__restrict__ rnk,
                                                         const JbHeader *hdr, T *__restrict__ X, T *__restrict__ W) {
  const T floor2 = (T)(Eps<T>::value * Eps<T>::value * hdr->fro2);
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < (int64_t)l * l;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(idx / l), r = (int)(idx - (int64_t)c * l);
    const T s = nrm[c];
    const int64_t dst = (int64_t)r * l + rnk[c];
    X[dst] = (s * s > floor2) ? Mt[idx] / s : (T)0;
    W[dst] = Jt[idx];
  }
}

constexpr int kJbMaxSweeps = 24;

// block width for the panel kernel: 2b columns of length l plus T must fit in LDS
static int jb_block_width(const rsvd_ctx *ctx, rsvd_dtype dtype, int64_t l) {
  const size_t es = dtype_size(dtype);
  for (int b = 32; b >= 8; b -= 8) {
    const size_t need = ((size_t)(2 * b) * (size_t)(l | 1) + (size_t)(2 * b) * ((2 * b) | 1)) * es + 1024;
    if (need <= ctx->lds_per_block) return b;
  }
  return 0;
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

// Scratch of the block path: header, Mt, Jt, norms, ranks.
size_t jacobi_scratch_bytes(const rsvd_ctx *ctx, rsvd_dtype dtype, int64_t l) {
  if (l <= jacobi_max_lds_order(ctx, dtype)) return 0;
  if (jb_block_width(ctx, dtype, l) == 0) return 0;          // unsupported order
  const size_t es = dtype_size(dtype);
  return align_up(sizeof(JbHeader), 256) + 2 * align_up((size_t)l * l * es, 256) + align_up((size_t)l * es, 256) +
         align_up((size_t)l * sizeof(int), 256);
}

template <typename T>
static hipError_t jacobi_block_launch(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype dtype, int l, const double *M,
                                      T *sigma, T *X, T *W, DevInfo *info, char *scratch) {
  const int b = jb_block_width(ctx, dtype, l);
  if (b == 0) return hipErrorNotSupported;
  const size_t es = sizeof(T);
  JbHeader *hdr = reinterpret_cast<JbHeader *>(scratch);
  char *p = scratch + align_up(sizeof(JbHeader), 256);
  T *Mt = reinterpret_cast<T *>(p); p += align_up((size_t)l * l * es, 256);
  T *Jt = reinterpret_cast<T *>(p); p += align_up((size_t)l * l * es, 256);
  T *nrm = reinterpret_cast<T *>(p); p += align_up((size_t)l * es, 256);
  int *rnk = reinterpret_cast<int *>(p);
  const int nblk = (l + b - 1) / b;
  const int nblk2 = nblk + (nblk & 1);
  const size_t lds = ((size_t)(2 * b) * (size_t)(l | 1) + (size_t)(2 * b) * ((2 * b) | 1)) * es;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&jb_panel_kernel<T, 32>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 512);
    (void)hipGetLastError();
    attr_set = true;
  }
  ProfScope ps(ctx, s, PK_JACOBI);
  hipLaunchKernelGGL((jb_init_kernel<T>), dim3(1), dim3(1024), 0, s, M, l, Mt, Jt, hdr);
  for (int sweep = 0; sweep < kJbMaxSweeps; ++sweep)
    for (int round = 0; round < nblk2 - 1; ++round)
      hipLaunchKernelGGL((jb_panel_kernel<T, 32>), dim3(nblk2 / 2), dim3(1024), lds, s, Mt, Jt, l, b, nblk, round,
                         sweep, 2, hdr);
  hipLaunchKernelGGL((jb_norms_kernel<T>), dim3((l + 3) / 4), dim3(256), 0, s, Mt, l, nrm);
  hipLaunchKernelGGL((jb_rank_kernel<T>), dim3((l + 255) / 256), dim3(256), 0, s, nrm, l, rnk, sigma, hdr,
                     kJbMaxSweeps, info);
  hipLaunchKernelGGL((jb_scatter_kernel<T>), dim3(256), dim3(256), 0, s, Mt, Jt, l, nrm, rnk, hdr, X, W);
  return hipGetLastError();
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
  if (l > jacobi_max_lds_order(ctx, dtype)) {
    // block path: needs the fp64 input (the triangular factor) and its scratch
    const size_t need = jacobi_scratch_bytes(ctx, dtype, l);
    if (need == 0 || scratch == nullptr || scratch_bytes < need || !m_is_f64) return hipErrorNotSupported;
    if (dtype == RSVD_F32)
      return jacobi_block_launch<float>(ctx, s, dtype, (int)l, (const double *)M, (float *)sigma, (float *)X,
                                        (float *)W, info, (char *)scratch);
    return jacobi_block_launch<double>(ctx, s, dtype, (int)l, (const double *)M, (double *)sigma, (double *)X,
                                       (double *)W, info, (char *)scratch);
  }
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
