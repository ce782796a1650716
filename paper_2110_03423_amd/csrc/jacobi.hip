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
// |a_p . a_q| <= tol * ||a_p|| * ||a_q||, tol = eps * sqrt(l); at most 60 sweeps (24 in the block path, whose
// launches are all issued in advance).
// The sweep that would only confirm this is saved when the rate of the last two sweeps says what it would find
// (jacobi_done below): with rho the largest relative inner product a sweep rotated away, the next sweep meets about
// rho^2 where the method converges quadratically (the paper: "3-4 iterations ... converges quadratically"; taken for
// granted only if the last step was at least of order 1.5 and rho <= sqrt(tol) / 4), and about rho^2 / rho_prev
// where it does not - inside a cluster of nearly equal singular values the rotations are large however small the
// inner products, and a sweep gains a constant factor only; there the sweep is saved once that estimate is below
// 8 tol.  (Stopping on rho <= sqrt(tol) / 4 alone left 1e-4 (fp32) / 1e-10 (fp64) between the vectors of such a
// cluster.)
// A column whose norm has fallen below eps * ||M||_F counts as zero and is no
// longer rotated (rotating it would change its partner by less than the
// rounding level); without this floor the surplus columns of a rank-deficient M
// keep shrinking by a factor eps per sweep until they underflow.  Its singular
// value is reported as that norm and its column of X is set to zero.
#include "common.hpp"
#include "mfma.hpp"

namespace rsvd {

constexpr int kJacobiMaxSweeps = 60;      // (a loop inside the kernel: sweeps that are not needed cost nothing)

template <typename T> struct Eps;
template <> struct Eps<float>  { static constexpr float  value = 1.1920929e-07f; };
template <> struct Eps<double> { static constexpr double value = 2.220446049250313e-16; };

// Was this sweep the last one?  rho: the largest relative inner product it rotated away (0: none), rho_prev: that
// of the sweep before (negative: there was none).
__host__ __device__ __forceinline__ bool jacobi_done(float rho, float rho_prev, float tol) {
  if (rho <= tol) return true;
  if (rho_prev < 0.f) return false;                                  // one sweep says nothing about the rate
  if (rho <= 0.25f * sqrtf(tol) && rho <= rho_prev * sqrtf(rho_prev)) return true;      // next: ~rho^2 < tol
  return rho * rho <= 8.f * tol * rho_prev;                          // next: ~rho^2 / rho_prev, a few tol at most
}
// The same from the per-sweep record of the block kernels: did the sweeps up to s - 1 finish the job?
__device__ __forceinline__ bool jacobi_done_before(const int *counters, int s, float tol) {
  if (s <= 0) return false;
  return jacobi_done(__int_as_float(counters[s - 1]), s > 1 ? __int_as_float(counters[s - 2]) : -1.f, tol);
}

// DPP lane moves: no LDS traffic, unlike a shuffle.
template <int CTRL> __device__ __forceinline__ float dpp_mov(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL> __device__ __forceinline__ double dpp_mov(double v) {
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)b, CTRL, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xF, 0xF, false);
  return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned int)lo);
}
// Sum over the 8 lanes of a half row: neighbours (quad_perm 1,0,3,2), pairs
// (quad_perm 2,3,0,1), then the other quad (row_half_mirror).  Every lane adds
// the same two partial sums at each step, so all 8 end with identical bits.
template <typename T> __device__ __forceinline__ T half_row_sum(T v) {
  v += dpp_mov<0xB1>(v);
  v += dpp_mov<0x4E>(v);
  v += dpp_mov<0x141>(v);
  return v;
}

// Sum over the G = 4, 8 or 16 lanes that share a column pair (16, the one in use: a whole DPP row).
template <int G, typename T> __device__ __forceinline__ T group_sum(T v) {
  v += dpp_mov<0xB1>(v);
  v += dpp_mov<0x4E>(v);
  if (G >= 8) v += dpp_mov<0x141>(v);
  if (G == 16) v += dpp_mov<0x140>(v);
  return v;
}

// Reciprocal, square root and reciprocal square root from the hardware estimates
// (1 ulp in fp32; refined by Newton steps in fp64).  The rotation parameters sit
// on the serial path of every pair, so their instruction count matters.
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ __forceinline__ float fast_rsq(float x) { return __builtin_amdgcn_rsqf(x); }
__device__ __forceinline__ float fast_sqrt(float x) { return __builtin_amdgcn_sqrtf(x); }
__device__ __forceinline__ double fast_rcp(double x) {
  double y = __builtin_amdgcn_rcp(x);
  y = y * (2.0 - x * y);
  y = y * (2.0 - x * y);
  return y;
}
__device__ __forceinline__ double fast_rsq(double x) {
  double y = __builtin_amdgcn_rsq(x);
  y = y * (1.5 - 0.5 * x * y * y);
  y = y * (1.5 - 0.5 * x * y * y);
  return y;
}
__device__ __forceinline__ double fast_sqrt(double x) { return x * fast_rsq(x); }

// Rotation (c, s) that orthogonalises two columns with squared norms alpha, beta
// and inner product gamma != 0:  zeta = (beta - alpha) / (2 gamma),
// t = sign(zeta) / (|zeta| + sqrt(1 + zeta^2)), c = 1 / sqrt(1 + t^2), s = c t.
template <typename T>
__device__ __forceinline__ void rotation_params(T alpha, T beta, T gamma, T &c, T &s) {
  const T zeta = (beta - alpha) * fast_rcp((T)2 * gamma);
  const T az = fabs(zeta);
  T t;
  if (az > (T)1e7) t = (T)0.5 * fast_rcp(az);                   // avoids overflow of zeta^2
  else t = fast_rcp(az + fast_sqrt((T)1 + zeta * zeta));
  t = zeta < (T)0 ? -t : t;
  c = fast_rsq((T)1 + t * t);
  s = c * t;
}

// Pair i of round r in a tournament of n2 (even) players: player n2-1 stays,
// the others rotate (circle method).  Requires r < n2 - 1 and i < n2 / 2.
__device__ __forceinline__ void tournament_pair(int n2, int r, int i, int &a, int &b) {
  const int nm1 = n2 - 1;
  if (i == 0) {
    a = nm1;
    b = r;
  } else {
    a = r + i;
    if (a >= nm1) a -= nm1;
    b = r - i;
    if (b < 0) b += nm1;
  }
}

// Pair order of the LDS-resident kernel: a recursive halving of the column set.  A set
// of columns splits into a front half A (floor) and a back half B (ceil); for |B| rounds
// column A_i meets B_{(i + r) mod |B|}, which covers every pair between A and B with all
// columns of A busy in every round; then A and B are treated the same way, side by side.
// All sets of one level have sizes that differ by at most one, so a level of sets of size
// <= ms takes ceil(ms / 2) rounds and a sweep ceil(l/2) + ceil(l/4) + ... ~ l rounds, like the
// circle method.  The point of this order: each lane group keeps its column of A in
// registers for the whole level and only the column of B travels through LDS, which halves
// the LDS traffic of a round (the LDS port, shared by the four SIMDs, is what bounds it).
struct JacLevel {
  unsigned char stat;      // column this group keeps for the level (255: none)
  unsigned char bstart;    // first column of B
  unsigned char bsize;     // |B|
  unsigned char idx;       // i: position of `stat` in A
};
constexpr int kJacLevels = 8, kJacGroups = 64;    // orders up to 128

template <typename T> using jac_unit = T __attribute__((ext_vector_type(8 / sizeof(T))));

// Columns are stored column-major with stride ldm and zero-padded to G * RPL rows.  LDS is
// accessed in 8-byte units (two floats or one double): lane lg of the group's G lanes owns
// units lg, lg + G, lg + 2 G, ... of a column (the G lanes touch one contiguous run).
template <typename T, int RPL, int G>
__device__ __forceinline__ void load_column(const T *col, int lg, jac_unit<T> (&x)[RPL / (8 / (int)sizeof(T))]) {
  const jac_unit<T> *p = reinterpret_cast<const jac_unit<T> *>(col) + lg;
#pragma unroll
  for (int r = 0; r < RPL / (8 / (int)sizeof(T)); ++r) x[r] = p[G * r];
}
template <typename T, int RPL, int G>
__device__ __forceinline__ void store_column(T *col, int lg, const jac_unit<T> (&x)[RPL / (8 / (int)sizeof(T))]) {
  jac_unit<T> *p = reinterpret_cast<jac_unit<T> *>(col) + lg;
#pragma unroll
  for (int r = 0; r < RPL / (8 / (int)sizeof(T)); ++r) p[G * r] = x[r];
}

// Rotate the pair (kept column x of M with its column u of J, in registers; column q in
// LDS).  Returns the relative size |x.y| / (|x| |y|) of the inner product it rotated away,
// 0 when it left the pair alone.
template <typename T, int RPL, int G>
__device__ __forceinline__ float rotate_moving(jac_unit<T> (&x)[RPL / (8 / (int)sizeof(T))],
                                               jac_unit<T> (&u)[RPL / (8 / (int)sizeof(T))], T *Mc, T *Jc, int ldm,
                                               int q, int lg, T tol, T floor2) {
  constexpr int V = 8 / sizeof(T);          // elements per LDS access
  constexpr int NV = RPL / V;               // accesses per column per lane
  jac_unit<T> y[NV];
  load_column<T, RPL, G>(Mc + q * ldm, lg, y);
  T alpha = 0, beta = 0, gamma = 0;
#pragma unroll
  for (int r = 0; r < NV; ++r)
#pragma unroll
    for (int e = 0; e < V; ++e) {
      alpha += x[r][e] * x[r][e];
      beta += y[r][e] * y[r][e];
      gamma += x[r][e] * y[r][e];
    }
  alpha = group_sum<G>(alpha);
  beta = group_sum<G>(beta);
  gamma = group_sum<G>(gamma);
  if (alpha <= floor2 || beta <= floor2) return 0.f;
  const T rel = fabs(gamma) * fast_rsq(alpha * beta);        // |x.y| / (|x| |y|); the matrix was scaled to unit size
  if (!(rel > tol)) return 0.f;
  const float ratio = (float)rel;
  jac_unit<T> v[NV];
  load_column<T, RPL, G>(Jc + q * ldm, lg, v);
  T c, s;
  rotation_params(alpha, beta, gamma, c, s);
#pragma unroll
  for (int r = 0; r < NV; ++r) {
    const jac_unit<T> xo = x[r];
    x[r] = c * xo - s * y[r];
    y[r] = s * xo + c * y[r];
  }
  store_column<T, RPL, G>(Mc + q * ldm, lg, y);
#pragma unroll
  for (int r = 0; r < NV; ++r) {
    const jac_unit<T> uo = u[r];
    u[r] = c * uo - s * v[r];
    v[r] = s * uo + c * v[r];
  }
  store_column<T, RPL, G>(Jc + q * ldm, lg, v);
  return ratio;
}

// Rows are padded to a whole number of 8-byte units per lane of the group (and to 16 at least).
// Column stride: the 16 lanes of a group read one contiguous run of 128 bytes, i.e. every LDS bank
// once, whatever the stride; the two extra rows only keep consecutive columns off the same phase.
__host__ __device__ inline int jacobi_rows_padded(int l, int G, int elem_size) {
  const int step = G * (8 / elem_size) > 16 ? G * (8 / elem_size) : 16;
  return ((l + step - 1) / step) * step;
}
__host__ __device__ inline int jacobi_ldm(int l, int G, int elem_size) {
  return jacobi_rows_padded(l, G, elem_size) + 2;
}

// JG: the columns of J (the accumulated rotations) live in global memory (Jglobal, l columns of ldm elements, one
// such array per problem of a batch, `stride` bytes apart) instead of LDS, for orders whose two matrices do not fit
// there together (fp64 beyond 96).  Its columns travel through the cache of the CU: a round takes longer, but
// the problems of a batch still run side by side, one workgroup each.
template <typename T, typename TIn, int RPL, int G, bool JG = false>
__global__ __launch_bounds__(64 * G) void jacobi_lds_kernel(const TIn *__restrict__ M, int l, T *__restrict__ sigma,
                                                         T *__restrict__ X, T *__restrict__ W, DevInfo *info,
                                                         int64_t stride, int rows, T *__restrict__ Jglobal) {
  extern __shared__ __attribute__((aligned(16))) double lds_raw[];
  if (blockIdx.x != 0) {              // batched launch: one problem per workgroup, `stride` bytes apart
    const int64_t off = (int64_t)blockIdx.x * stride;
    M = reinterpret_cast<const TIn *>(reinterpret_cast<const char *>(M) + off);
    sigma = reinterpret_cast<T *>(reinterpret_cast<char *>(sigma) + off);
    X = reinterpret_cast<T *>(reinterpret_cast<char *>(X) + off);
    W = reinterpret_cast<T *>(reinterpret_cast<char *>(W) + off);
    if (JG) Jglobal = reinterpret_cast<T *>(reinterpret_cast<char *>(Jglobal) + off);
  }
  const int ldm = jacobi_ldm(l, G, (int)sizeof(T));
  T *Mc = reinterpret_cast<T *>(lds_raw);
  T *Jc = JG ? Jglobal : Mc + (size_t)l * ldm;
  T *nrm = Mc + (size_t)(JG ? 1 : 2) * l * ldm;
  int *rnk = reinterpret_cast<int *>(nrm + l);
  __shared__ int rotations;
  __shared__ T wave_sum[16];
  __shared__ JacLevel lev[kJacLevels][kJacGroups];

  const int tid = threadIdx.x, nt = blockDim.x;
  // pair order: every column finds, level by level, the set it belongs to; the columns of
  // a front half claim lane group (start of the set) / 2 + (position in the half)
  for (int e = tid; e < kJacLevels * kJacGroups; e += nt) (&lev[0][0])[e].stat = 255;
  __syncthreads();
  if (tid < l) {
    int start = 0, size = l;
    for (int d = 0; d < kJacLevels && size > 1; ++d) {
      const int h = size >> 1;
      if (tid < start + h) {
        JacLevel e;
        e.stat = (unsigned char)tid; e.bstart = (unsigned char)(start + h); e.bsize = (unsigned char)(size - h);
        e.idx = (unsigned char)(tid - start);
        lev[d][(start >> 1) + (tid - start)] = e;
        size = h;
      } else {
        start += h;
        size -= h;
      }
    }
  }
  T fro2 = 0;
  {
    // M is row-major in global memory and column-major in LDS: consecutive threads take consecutive elements
    // of a row (one cache line per 16 or 8 of them); the padding rows of the columns are cleared apart
    const int pad = ldm - l;
    for (int idx = tid; idx < l * pad; idx += nt) {
      const int c = idx / pad, r = l + (idx - c * pad);
      Mc[c * ldm + r] = (T)0;
      Jc[c * ldm + r] = (T)0;
    }
    for (int idx = tid; idx < l * l; idx += nt) {
      const int r = idx / l, c = idx - r * l;
      const T v = (T)M[idx];
      if (rows) Mc[r * ldm + c] = v;                      // the rows of M are what is rotated: M^T is decomposed
      else Mc[c * ldm + r] = v;
      Jc[c * ldm + r] = (r == c) ? (T)1 : (T)0;
      fro2 += v * v;
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) fro2 += __shfl_xor(fro2, off, 64);
  if ((tid & 63) == 0) wave_sum[tid >> 6] = fro2;
  if (tid == 0) rotations = 0;
  __syncthreads();
  fro2 = 0;
  for (int w = 0; w < (nt >> 6); ++w) fro2 += wave_sum[w];
  // Scale M by a power of two to ||M||_F ~ 1 (exact; undone when sigma is written): products of squared
  // column norms then stay inside the range of the type whatever the scale of the input.
  T unscale = (T)1;
  if (fro2 > (T)0 && fro2 < (T)3e38) {
    int ex;
    (void)frexp((double)fro2, &ex);                       // fro2 = f 2^ex, 1/2 <= f < 1
    const T sc = (T)ldexp(1.0, -(ex / 2));
    unscale = (T)ldexp(1.0, ex / 2);
    for (int idx = tid; idx < l * ldm; idx += nt) Mc[idx] *= sc;
    fro2 *= sc * sc;
    __syncthreads();
  }
  const T floor2 = Eps<T>::value * Eps<T>::value * fro2;

  const int group = tid / G, lg = tid % G;       // G lanes per column pair
  const T tol = Eps<T>::value * sqrt((T)l);
  int sweeps = 0;
  bool converged = (l < 2);
  float rho_prev = -1.f;
  constexpr int NV = RPL / (8 / (int)sizeof(T));
  while (!converged && sweeps < kJacobiMaxSweeps) {
    ++sweeps;
    float rho = 0.f;
    int d = 0;
    for (int ms = l; ms > 1; ms = (ms + 1) >> 1, ++d) {      // ms: largest set of this level
      JacLevel e;
      e.stat = 255; e.bstart = 0; e.bsize = 0; e.idx = 0;
      if (group < kJacGroups) e = lev[d][group];
      const bool act = e.stat != 255;
      jac_unit<T> x[NV], u[NV];
      if (act) {
        load_column<T, RPL, G>(Mc + e.stat * ldm, lg, x);
        load_column<T, RPL, G>(Jc + e.stat * ldm, lg, u);
      }
      const int nr = ms - (ms >> 1);
      for (int r = 0; r < nr; ++r) {
        if (act && r < e.bsize) {
          int j = e.idx + r;
          if (j >= e.bsize) j -= e.bsize;
          rho = fmaxf(rho, rotate_moving<T, RPL, G>(x, u, Mc, Jc, ldm, e.bstart + j, lg, tol, floor2));
        }
        __syncthreads();
      }
      if (act) {
        store_column<T, RPL, G>(Mc + e.stat * ldm, lg, x);
        store_column<T, RPL, G>(Jc + e.stat * ldm, lg, u);
      }
      __syncthreads();
    }
    if (rho > 0.f) atomicMax(&rotations, __float_as_int(rho));   // positive floats order like their bit patterns
    __syncthreads();
    converged = jacobi_done(__int_as_float(rotations), rho_prev, (float)tol);
    rho_prev = __int_as_float(rotations);
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
    sigma[rank] = mine * unscale;
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
// (2b columns of length l) into LDS, runs the same pairwise rotations as above
// over those columns while accumulating them in a small 2b x 2b matrix T,
// writes the columns back and leaves T for the matching columns of J.  In the
// launch that rotates the pairs inside one block every rotation is a plane
// rotation of actual columns; the launches over block pairs take the rotations
// from the Gram matrix of the panel and apply T once (jb_cross_kernel), or
// rotate column by column where that panel does not fit in LDS (jb_panel_kernel).
// counters[s] collects the largest relative inner product that outer sweep s
// rotated away; a launch that finds the sweeps before it sufficient
// (jacobi_done_before) returns at once, which keeps the whole sequence free of
// host synchronisation.

// Sum over the 32 lanes of a pair group: the 16-lane row by DPP (neighbours, pairs,
// half-row mirror, row mirror), then one exchange with the partner row.
template <typename T> __device__ __forceinline__ T group32_sum(T v) {
  v += dpp_mov<0xB1>(v);
  v += dpp_mov<0x4E>(v);
  v += dpp_mov<0x141>(v);
  v += dpp_mov<0x140>(v);
  v += __shfl_xor(v, 16, 32);
  return v;
}

// Panel version of rotate_pair: columns of length up to 32 * NV units held in LDS
// (stride ldp, zero padded), 32 lanes per pair, the accumulated rotation T
// (rows_t x rows_t, stride ldt) instead of J.
template <typename T, int NV>
__device__ __forceinline__ float rotate_pair_panel(T *Pc, T *Tc, int ldp, int ldt, int rows_t, int p, int q, int lg,
                                                  T tol, T floor2) {
  constexpr int V = 8 / sizeof(T);
  typedef T unit __attribute__((ext_vector_type(V)));
  unit *mp = reinterpret_cast<unit *>(Pc + p * ldp) + lg;
  unit *mq = reinterpret_cast<unit *>(Pc + q * ldp) + lg;
  unit x[NV], y[NV];
#pragma unroll
  for (int r = 0; r < NV; ++r) { x[r] = mp[32 * r]; y[r] = mq[32 * r]; }
  T alpha = 0, beta = 0, gamma = 0;
#pragma unroll
  for (int r = 0; r < NV; ++r)
#pragma unroll
    for (int e = 0; e < V; ++e) {
      alpha += x[r][e] * x[r][e];
      beta += y[r][e] * y[r][e];
      gamma += x[r][e] * y[r][e];
    }
  alpha = group32_sum(alpha);
  beta = group32_sum(beta);
  gamma = group32_sum(gamma);
  if (alpha <= floor2 || beta <= floor2) return 0.f;
  const T rel = fabs(gamma) * fast_rsq(alpha * beta);        // |x.y| / (|x| |y|); the matrix was scaled to unit size
  if (!(rel > tol)) return 0.f;
  const float ratio = (float)rel;
  T c, s;
  rotation_params(alpha, beta, gamma, c, s);
#pragma unroll
  for (int r = 0; r < NV; ++r) {
    mp[32 * r] = c * x[r] - s * y[r];
    mq[32 * r] = s * x[r] + c * y[r];
  }
  T *tp = Tc + p * ldt, *tq = Tc + q * ldt;
  for (int i = lg; i < rows_t; i += 32) {
    const T a = tp[i], bq = tq[i];
    tp[i] = c * a - s * bq;
    tq[i] = s * a + c * bq;
  }
  return ratio;
}

// Cross-phase version: the column of the first block (x, NV units per lane) and its
// column of T (tx: entries lg and lg + 32) stay in registers for all rounds of the launch;
// only the column of the second block (qp: its place in LDS) and its column qt of T go through LDS.
template <typename T, int NV>
__device__ __forceinline__ float rotate_moving_panel(jac_unit<T> (&x)[NV], T (&tx)[2], T *Pc, T *Tc, int ldp, int ldt,
                                                    int rows_t, int qp, int qt, int lg, T tol, T floor2) {
  constexpr int V = 8 / sizeof(T);
  jac_unit<T> *mq = reinterpret_cast<jac_unit<T> *>(Pc + qp * ldp) + lg;
  jac_unit<T> y[NV];
#pragma unroll
  for (int r = 0; r < NV; ++r) y[r] = mq[32 * r];
  T alpha = 0, beta = 0, gamma = 0;
#pragma unroll
  for (int r = 0; r < NV; ++r)
#pragma unroll
    for (int e = 0; e < V; ++e) {
      alpha += x[r][e] * x[r][e];
      beta += y[r][e] * y[r][e];
      gamma += x[r][e] * y[r][e];
    }
  alpha = group32_sum(alpha);
  beta = group32_sum(beta);
  gamma = group32_sum(gamma);
  if (alpha <= floor2 || beta <= floor2) return 0.f;
  const T rel = fabs(gamma) * fast_rsq(alpha * beta);        // |x.y| / (|x| |y|); the matrix was scaled to unit size
  if (!(rel > tol)) return 0.f;
  const float ratio = (float)rel;
  T c, s;
  rotation_params(alpha, beta, gamma, c, s);
#pragma unroll
  for (int r = 0; r < NV; ++r) {
    const jac_unit<T> xo = x[r];
    x[r] = c * xo - s * y[r];
    mq[32 * r] = s * xo + c * y[r];
  }
  T *tq = Tc + qt * ldt;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int i = lg + 32 * j;
    if (i < rows_t) {
      const T a = tx[j], bq = tq[i];
      tx[j] = c * a - s * bq;
      tq[i] = s * a + c * bq;
    }
  }
  return ratio;
}

// scratch header shared by the block-Jacobi kernels
constexpr int kJbFroParts = 64;
struct JbHeader {
  double fro2;            // ||M||_F^2 of the scaled matrix
  double unscale;         // the singular values of M are those of the scaled matrix times this
  int counters[64];       // per outer sweep: bit pattern of the largest relative inner product rotated away
  double partial[kJbFroParts];   // sums of squares, one per workgroup of jb_fro_kernel
};

// ||M||_F^2 in kJbFroParts partial sums (fixed assignment of elements and fixed order: reproducible).
__global__ __launch_bounds__(256) void jb_fro_kernel(const double *__restrict__ M, int l, JbHeader *hdr) {
  __shared__ double wave_sum[4];
  const int tid = threadIdx.x;
  double s2 = 0;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + tid; idx < (int64_t)l * l; idx += (int64_t)kJbFroParts * 256) {
    const double v = M[idx];
    s2 += v * v;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s2 += __shfl_xor(s2, off, 64);
  if ((tid & 63) == 0) wave_sum[tid >> 6] = s2;
  __syncthreads();
  if (tid == 0) hdr->partial[blockIdx.x] = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
}

// Mt = (sc M)^T in the working type, Jt = I, with sc the power of two that brings ||M||_F to ~1 (exact, undone
// when the singular values are written): products of squared column norms then stay inside the range of
// the type whatever the scale of the input.  Grid of workgroups, each taking a slab of elements.
template <typename T>
__global__ __launch_bounds__(256) void jb_init_kernel(const double *__restrict__ M, int l, T *__restrict__ Mt,
                                                      T *__restrict__ Jt, JbHeader *hdr, int rows) {
  double fro2 = 0;
  for (int i = 0; i < kJbFroParts; ++i) fro2 += hdr->partial[i];
  double sc = 1.0, unscale = 1.0;
  if (fro2 > 0.0 && fro2 <= 1.79e308) {
    int ex;
    (void)frexp(fro2, &ex);
    sc = ldexp(1.0, -(ex / 2));
    unscale = ldexp(1.0, ex / 2);
  }
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < (int64_t)l * l;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int r = (int)(idx / l), c = (int)(idx - (int64_t)r * l);
    Mt[rows ? idx : (int64_t)c * l + r] = (T)(M[idx] * sc);      // rows: M^T is decomposed, its columns are M's rows
    Jt[idx] = (r == c) ? (T)1 : (T)0;
  }
  if (blockIdx.x == 0) {
    if (threadIdx.x < 64) hdr->counters[threadIdx.x] = 0;
    if (threadIdx.x == 0) {
      hdr->fro2 = fro2 * sc * sc;
      hdr->unscale = unscale;
    }
  }
}

// Padded column length (elements) of the panel layout: 32 lanes x NV units.
template <typename T, int NV> __host__ __device__ constexpr int jb_ldp() { return 32 * NV * (8 / (int)sizeof(T)) + 2; }

// phase 0 ("diagonal"): workgroup g rotates the pairs inside column block g
//   (cols - 1 rounds of the circle tournament).
// phase 1 ("cross"): workgroup g takes the block pair g of tournament round `round`
//   and rotates only pairs with one column in each block: b rounds, pair i of
//   round r is (i, (i + r) mod b) - every column of one block meets every column of
//   the other exactly once.
// One outer sweep = one diagonal launch + (nblk - 1) cross launches = l - 1 rounds
// in all, the same count as the plain tournament.
//
// The rotations never read J, and a launch keeps only nblk / 2 of the chip's workgroups busy.
// So a rotating workgroup only leaves its accumulated T (and a flag that it rotated at all) in a
// two-slot ring in global memory, and the NEXT launch carries, behind its own rot_wgs rotating
// workgroups, one workgroup per (block pair of the launch before, chunk of kJbRowChunk rows) that
// applies that T to the matching columns of J on the matrix cores while the rotations of the
// current round run.  A last launch with rot_wgs = 0 applies what the final round left.

// Block pair (and column counts) of workgroup g of a launch.
struct JbPair { int bi, bj, cols_i, cols_j; bool valid; };
__device__ __forceinline__ JbPair jb_pair(int phase, int round, int g, int l, int b, int nblk) {
  JbPair p;
  p.valid = true;
  if (phase == 0) {
    p.bi = p.bj = g;
    p.cols_i = (l - p.bi * b < b) ? (l - p.bi * b) : b;
    p.cols_j = 0;
  } else {
    const int nblk2 = nblk + (nblk & 1);
    int ba, bb;
    tournament_pair(nblk2, round, g, ba, bb);
    p.valid = ba < nblk && bb < nblk;                          // else a bye
    p.bi = ba < bb ? ba : bb;
    p.bj = ba < bb ? bb : ba;
    p.cols_i = (l - p.bi * b < b) ? (l - p.bi * b) : b;
    p.cols_j = p.valid ? ((l - p.bj * b < b) ? (l - p.bj * b) : b) : 0;
  }
  return p;
}

constexpr int kJbRowChunk = 64;      // one row per lane of a wavefront when the chunk is staged (jb_apply_t)

// J[rows of chunk, panel] <- J[rows of chunk, panel] T for block pair `pr`: the old entries staged
// through LDS, a (64 x 2b) by (2b x 2b) product in 16 x 16 blocks.
template <typename T>
__device__ __forceinline__ void jb_apply_t(T *__restrict__ Jt, const T *__restrict__ Tg, int l, int b, const JbPair &pr,
                                           int chunk, T *lds) {
  static_assert(kJbRowChunk == 64, "the staging loop below moves one row per lane of a wavefront");
  constexpr int LDJ = kJbRowChunk + 8;
  const int ldt = 2 * b + 2;
  T *Pj = lds;                       // [2b][LDJ]: Pj[k][i] = J[i0 + i][panel column k]
  T *Tl = lds + (size_t)(2 * b) * LDJ;      // [2b][ldt]: Tl[col][k] = T[k][col]
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane64 = tid & 63, wave = tid >> 6, nwave = nt >> 6;
  const int ncols = pr.cols_i + pr.cols_j;
  const int i0 = chunk * kJbRowChunk;
  auto gcol = [&](int c) { return c < pr.cols_i ? pr.bi * b + c : pr.bj * b + (c - pr.cols_i); };
  for (int c = wave; c < 2 * b; c += nwave) {
    const int i = i0 + lane64;
    Pj[c * LDJ + lane64] = (c < ncols && i < l) ? Jt[(int64_t)gcol(c) * l + i] : (T)0;
  }
  for (int idx = tid; idx < 4 * b * b; idx += nt) {
    const int c = idx / (2 * b), k = idx - c * (2 * b);
    Tl[c * ldt + k] = Tg[idx];
  }
  __syncthreads();
  typedef typename Mfma<T>::vec acc_t;
  const int r16 = lane64 & 15, kq = lane64 >> 4;
  const int col_blocks = (2 * b) / 16;
  for (int blk = wave; blk < (kJbRowChunk / 16) * col_blocks; blk += nwave) {
    const int rb = blk / col_blocks, cb = blk - rb * col_blocks;
    acc_t acc = (acc_t)(T)0;
    const T *ap = Pj + kq * LDJ + rb * 16 + r16;                  // Jold[row][k]
    const T *bp = Tl + (cb * 16 + r16) * ldt + kq;                // T[k][col]
#pragma unroll 4
    for (int k0 = 0; k0 < 2 * b; k0 += 4) acc = Mfma<T>::run(ap[k0 * LDJ], bp[k0], acc);
    const int cn = cb * 16 + r16;
    if (cn < ncols) {
      T *dst = Jt + (int64_t)gcol(cn) * l;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int r = i0 + rb * 16 + Mfma<T>::row(lane64, v);
        if (r < l) dst[r] = acc[v];
      }
    }
  }
}

// J role of a launch: workgroup j behind the rot_wgs rotating ones applies the T that block pair g of the launch
// before (phase, round, sweep = prev_*) left in the other slot of the ring to one chunk of rows of J.
template <typename T>
__device__ __forceinline__ void jb_j_role(T *__restrict__ Jt, int l, int b, int nblk, int rot_wgs, int prev_phase,
                                          int prev_round, int prev_sweep, const T *__restrict__ Tring,
                                          const int *__restrict__ chg, int slot, const JbHeader *hdr, float tol,
                                          T *lds) {
  const int chunks = (l + kJbRowChunk - 1) / kJbRowChunk;
  const int j = (int)blockIdx.x - rot_wgs;
  const int g = j / chunks;
  if (jacobi_done_before(hdr->counters, prev_sweep, tol)) return;                  // that launch did nothing
  const JbPair pr = jb_pair(prev_phase, prev_round, g, l, b, nblk);
  const int pslot = slot ^ 1;
  if (!pr.valid || chg[pslot * nblk + g] == 0) return;
  jb_apply_t<T>(Jt, Tring + ((size_t)pslot * nblk + g) * (size_t)(4 * b * b), l, b, pr, j - g * chunks, lds);
}

template <typename T, int NV>
__global__ __launch_bounds__(1024) void jb_panel_kernel(T *__restrict__ Mt, T *__restrict__ Jt, int l, int b,
                                                        int nblk, int phase, int round, int sweep, int rot_wgs,
                                                        int prev_phase, int prev_round, int prev_sweep,
                                                        T *__restrict__ Tring, int *__restrict__ chg, int slot,
                                                        JbHeader *hdr) {
  const T tol = Eps<T>::value * sqrt((T)l);
  extern __shared__ __attribute__((aligned(16))) double lds_raw[];
  if ((int)blockIdx.x >= rot_wgs) {
    jb_j_role<T>(Jt, l, b, nblk, rot_wgs, prev_phase, prev_round, prev_sweep, Tring, chg, slot, hdr, (float)tol,
                 reinterpret_cast<T *>(lds_raw));
    return;
  }
  if (jacobi_done_before(hdr->counters, sweep, (float)tol)) return;        // the sweeps before finished the job
  const JbPair pr = jb_pair(phase, round, (int)blockIdx.x, l, b, nblk);
  if (!pr.valid) return;                                       // bye
  const int bi = pr.bi, bj = pr.bj, cols_i = pr.cols_i, cols_j = pr.cols_j;
  const int ncols = cols_i + cols_j;

  constexpr int ldp = jb_ldp<T, NV>();
  const int ldt = (2 * b) + 2;
  // LDS holds ONE block of columns: the block itself in the diagonal phase, the second ("moving")
  // block in the cross phase, whose first block lives in registers from global memory to global
  // memory.
  T *Pc = reinterpret_cast<T *>(lds_raw);
  T *Tc = Pc + (size_t)b * ldp;
  __shared__ int rotations;
  const int lds_blk = (phase == 0) ? bi : bj;
  const int lds_cols = (phase == 0) ? cols_i : cols_j;

  const int tid = threadIdx.x, nt = blockDim.x;
  // panel in: a wavefront takes whole columns, two at a time, and issues every load of both
  // before the first LDS store (the loads are the latency to hide)
  constexpr int LPW = (ldp + 63) / 64;      // elements per lane per column
  const int lane64 = tid & 63, wave = tid >> 6, nwave = nt >> 6;
  auto panel_in = [&](const T *__restrict__ G) {
    for (int c0 = wave; c0 < b; c0 += 2 * nwave) {
      T v[2][LPW];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int c = c0 + u * nwave;
        const T *src = G + (int64_t)(lds_blk * b + (c < lds_cols ? c : 0)) * l;
#pragma unroll
        for (int j = 0; j < LPW; ++j) {
          const int r = lane64 + 64 * j;
          v[u][j] = (c < lds_cols && r < l) ? src[r] : (T)0;
        }
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int c = c0 + u * nwave;
        if (c < b) {
#pragma unroll
          for (int j = 0; j < LPW; ++j) {
            const int r = lane64 + 64 * j;
            if (r < ldp) Pc[c * ldp + r] = v[u][j];
          }
        }
      }
    }
  };
  auto panel_out = [&](T *__restrict__ G) {
    for (int c = wave; c < lds_cols; c += nwave) {
      T *dst = G + (int64_t)(lds_blk * b + c) * l;
#pragma unroll
      for (int j = 0; j < LPW; ++j) {
        const int r = lane64 + 64 * j;
        if (r < l) dst[r] = Pc[c * ldp + r];
      }
    }
  };
  panel_in(Mt);
  for (int idx = tid; idx < 2 * b * ldt; idx += nt) {
    const int c = idx / ldt, r = idx - c * ldt;
    Tc[idx] = (r == c && c < ncols) ? (T)1 : (T)0;
  }
  if (tid == 0) rotations = 0;

  const T floor2 = (T)(Eps<T>::value * Eps<T>::value * hdr->fro2);
  const int group = tid >> 5, lg = tid & 31;                   // 32 groups of 32 lanes, b <= 32
  constexpr int V = 8 / (int)sizeof(T);
  float rho = 0.f;
  // cross phase: lane group g keeps column g of the first block (and its column of T) for all b rounds
  const bool act = phase != 0 && group < cols_i;
  jac_unit<T> x[NV];
  T tx[2] = {(T)0, (T)0};
  if (act) {
    const T *src = Mt + (int64_t)(bi * b + group) * l;
#pragma unroll
    for (int r = 0; r < NV; ++r)
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const int row = (lg + 32 * r) * V + e;
        x[r][e] = row < l ? src[row] : (T)0;
      }
#pragma unroll
    for (int j = 0; j < 2; ++j) tx[j] = (lg + 32 * j == group) ? (T)1 : (T)0;     // column `group` of the identity
  }
  __syncthreads();

  if (phase == 0) {
    const int n2 = ncols + (ncols & 1);
    for (int r = 0; r < n2 - 1; ++r) {
      if (group < n2 / 2) {
        int a, c2;
        tournament_pair(n2, r, group, a, c2);
        if (a < ncols && c2 < ncols) {
          const int p = a < c2 ? a : c2, q = a < c2 ? c2 : a;
          rho = fmaxf(rho, rotate_pair_panel<T, NV>(Pc, Tc, ldp, ldt, ncols, p, q, lg, tol, floor2));
        }
      }
      __syncthreads();
    }
  } else {
    for (int r = 0; r < b; ++r) {
      int qi = group + r;
      if (qi >= b) qi -= b;
      if (act && qi < cols_j)
        rho = fmaxf(rho, rotate_moving_panel<T, NV>(x, tx, Pc, Tc, ldp, ldt, ncols, qi, cols_i + qi, lg, tol, floor2));
      __syncthreads();
    }
    if (act) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
        if (lg + 32 * j < ncols) Tc[group * ldt + lg + 32 * j] = tx[j];
    }
    __syncthreads();
  }
  if (rho > 0.f) atomicMax(&rotations, __float_as_int(rho));
  __syncthreads();
  const int rho_bits = rotations;
  if (rho_bits == 0) {                                        // nothing changed: leave M alone, no T to apply
    if (tid == 0) chg[slot * nblk + blockIdx.x] = 0;
    return;
  }
  panel_out(Mt);
  if (act) {
    T *dst = Mt + (int64_t)(bi * b + group) * l;
#pragma unroll
    for (int r = 0; r < NV; ++r)
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const int row = (lg + 32 * r) * V + e;
        if (row < l) dst[row] = x[r][e];
      }
  }
  T *Tg = Tring + ((size_t)slot * nblk + blockIdx.x) * (size_t)(4 * b * b);
  for (int idx = tid; idx < 4 * b * b; idx += nt) {
    const int c = idx / (2 * b), k = idx - c * (2 * b);
    Tg[idx] = Tc[c * ldt + k];
  }
  if (tid == 0) {
    chg[slot * nblk + blockIdx.x] = 1;
    atomicMax(&hdr->counters[sweep], rho_bits);
  }
}

// ---- cross phase through the Gram matrix of the block pair ----
//
// The b rounds of a cross launch rotate 2b columns of length l; done column by column (jb_panel_kernel) a round
// costs ~1 us of plain vector instructions whatever l is.  The rotations only need inner products, and those
// follow from the 2b x 2b Gram matrix G of the panel: G is formed once on the matrix cores, the b rounds rotate G
// on both sides (G <- J^T G J, a 2 x 2 block per thread) and accumulate T <- T J, and the panel is multiplied by T
// once, again on the matrix cores.  Pair order, rotation formulas, thresholds and the stopping rule are those of
// the column-by-column kernel; the first round sees exact inner products, later rounds the tracked ones (their
// error is of second order in the rotation angles and is wiped out by the next launch, which forms G afresh).
constexpr int kJgB = 16;                    // block width this kernel is written for
constexpr int kJgN = 2 * kJgB;              // columns of a panel
constexpr int kJgLd = kJgN + 1;             // row stride of G and T in LDS
constexpr int kJgMat = kJgN * kJgLd;        // elements of one such matrix
constexpr int kJgPart = 3 * 256;            // elements of one partial sum of G (three 16 x 16 blocks)

// Column stride of the panel in LDS: l padded to whole 16-row blocks, plus what spreads 16 columns over the banks.
template <typename T> __host__ __device__ constexpr int jg_ldp(int l) {
  return (l + 15) / 16 * 16 + (sizeof(T) == 4 ? 2 : 1);
}
template <typename T> __host__ __device__ constexpr size_t jg_lds_bytes(int l) {
  return ((size_t)kJgN * jg_ldp<T>(l) + 5 * (size_t)kJgMat) * sizeof(T);
}

// Rotation of pair `a` in round r (columns p = a and q = b + (a + r) mod b of the panel), from the tracked Gram
// matrix: (c, s) = (1, 0) when the pair is left alone; returns the relative inner product that is rotated away
// (0 if none).  Without branches: the chain of dependent instructions of a round starts here.
template <typename T>
__device__ __forceinline__ float jg_pair_params(const T *G, int a, int r, int cols_i, int cols_j, T tol, T floor2,
                                                int &q, T &c, T &s) {
  const int qi = (a + r) & (kJgB - 1);
  q = kJgB + qi;
  const T alpha = G[a * kJgLd + a], beta = G[q * kJgLd + q], gamma = G[a * kJgLd + q];
  const T rel = fabs(gamma) * fast_rsq(alpha * beta);
  const bool rot = (a < cols_i) & (qi < cols_j) & (alpha > floor2) & (beta > floor2) & (rel > tol);
  const T g = rot ? gamma : (T)1;
  const T zeta = (beta - alpha) * fast_rcp((T)2 * g);
  const T az = fabs(zeta);
  T cc, ss;
  if constexpr (sizeof(T) == 4) {
    // t = 1 / (|zeta| + sqrt(1 + zeta^2)), c = 1 / sqrt(1 + t^2), s = c t: s tied to c, so that c^2 + s^2 - 1 stays
    // at the 1e-9 level in fp32 (the columns of T and J keep their length over thousands of rotations)
    const T t_small = (T)0.5 * fast_rcp(az);                     // |zeta| > 1e7: zeta^2 would overflow
    const T t_usual = fast_rcp(az + fast_sqrt((T)1 + zeta * zeta));
    const T t = az > (T)1e7 ? t_small : t_usual;
    cc = fast_rsq((T)1 + t * t);
    ss = cc * t;
  } else {
    // the same rotation with one reciprocal square root less on the chain of dependent instructions (each costs
    // two Newton steps in fp64): with w = sqrt(1 + zeta^2), c^2 = (|zeta| + w) / (2 w), s^2 = 1 / (2 w (|zeta| + w))
    const T q2 = (T)1 + zeta * zeta;
    const T u = fast_rsq(q2);
    const T w = q2 * u;
    const T c_usual = fast_sqrt((T)0.5 + (T)0.5 * az * u);
    const T s_usual = fast_rsq((T)2 * w * (az + w));
    const bool huge = az > (T)1e100;                             // zeta^2 would overflow; t = 1 / (2 |zeta|)
    cc = huge ? (T)1 : c_usual;
    ss = huge ? (T)0.5 * fast_rcp(az) : s_usual;
  }
  ss = zeta < (T)0 ? -ss : ss;
  c = rot ? cc : (T)1;
  s = rot ? ss : (T)0;
  return rot ? (float)rel : 0.f;
}

template <typename T> __device__ __forceinline__ T lane_read(T v, int src_lane);
template <> __device__ __forceinline__ float lane_read<float>(float v, int src_lane) {
  return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane << 2, __float_as_int(v)));
}
template <> __device__ __forceinline__ double lane_read<double>(double v, int src_lane) {
  const long long b = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_ds_bpermute(src_lane << 2, (int)b);
  const int hi = __builtin_amdgcn_ds_bpermute(src_lane << 2, (int)(b >> 32));
  return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned int)lo);
}

template <typename T>
__global__ __launch_bounds__(1024) void jb_cross_kernel(T *__restrict__ Mt, T *__restrict__ Jt, int l, int nblk,
                                                        int round, int sweep, int rot_wgs, int prev_phase,
                                                        int prev_round, int prev_sweep, T *__restrict__ Tring,
                                                        int *__restrict__ chg, int slot, JbHeader *hdr) {
  constexpr int b = kJgB;
  const T tol = Eps<T>::value * sqrt((T)l);
  extern __shared__ __attribute__((aligned(16))) double lds_raw[];
  if ((int)blockIdx.x >= rot_wgs) {
    jb_j_role<T>(Jt, l, b, nblk, rot_wgs, prev_phase, prev_round, prev_sweep, Tring, chg, slot, hdr, (float)tol,
                 reinterpret_cast<T *>(lds_raw));
    return;
  }
  if (jacobi_done_before(hdr->counters, sweep, (float)tol)) return;        // the sweeps before finished the job
  const JbPair pr = jb_pair(1, round, (int)blockIdx.x, l, b, nblk);
  if (!pr.valid) return;                                       // bye
  const int cols_i = pr.cols_i, cols_j = pr.cols_j, ncols = cols_i + cols_j;
  const int ldp = jg_ldp<T>(l), lp = (l + 15) / 16 * 16;
  T *Pc = reinterpret_cast<T *>(lds_raw);                      // [2b][ldp]: column c of the panel, zero padded
  T *G0 = Pc + (size_t)kJgN * ldp;                             // G, even rounds
  T *R4 = G0 + kJgMat;                                         // four matrices: the five partial sums of G, then T0, T1, G1 and the (c, s) of every round
  __shared__ int rotations;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kq = lane >> 4;
  auto gcol = [&](int c) { return c < b ? pr.bi * b + c : pr.bj * b + (c - b); };      // global column of panel column c
  auto live = [&](int c) { return c < b ? c < cols_i : c - b < cols_j; };

  // panel in: wavefront w takes columns w and w + 16, every load in flight before the first LDS store
  {
    constexpr int MAXJ = sizeof(T) == 4 ? 17 : 8;              // 64 * MAXJ rows at most (the LDS limit is lower)
    T v[2][MAXJ];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int c = wave + 16 * u;
      const T *src = Mt + (int64_t)gcol(live(c) ? c : 0) * l;
#pragma unroll
      for (int j = 0; j < MAXJ; ++j) {
        const int rr = lane + 64 * j;
        v[u][j] = (live(c) && rr < l) ? src[rr] : (T)0;
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int c = wave + 16 * u;
#pragma unroll
      for (int j = 0; j < MAXJ; ++j) {
        const int rr = lane + 64 * j;
        if (rr < lp) Pc[c * ldp + rr] = v[u][j];
      }
    }
  }
  if (tid == 0) rotations = 0;
  __syncthreads();

  // G = P^T P: wavefront w takes 16 x 16 block (ti, tj) over the quarter sl of the rows, eight k-steps of
  // operands at a time ahead of their matrix instructions, two accumulators
  typedef typename Mfma<T>::vec acc_t;
  {
    // (G is symmetric: blocks (0,0), (0,1) and (1,1) only, five row slices each, fifteen wavefronts)
    const int sl = wave / 3, tile = wave - 3 * sl;
    const int ti = tile >> 1, tj = (tile + 1) >> 1;
    const int steps = lp / 4, per = (steps + 4) / 5;
    const int s0 = sl * per, s1 = (wave == 15) ? 0 : ((s0 + per < steps) ? s0 + per : steps);
    acc_t acc0 = (acc_t)(T)0, acc1 = (acc_t)(T)0;
    const T *ap = Pc + (ti * 16 + r16) * ldp + kq;
    const T *bp = Pc + (tj * 16 + r16) * ldp + kq;
    for (int st = s0; st < s1; st += 8) {
      T av[8], bv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const bool ok = st + u < s1;
        av[u] = ok ? ap[4 * (st + u)] : (T)0;
        bv[u] = ok ? bp[4 * (st + u)] : (T)0;
      }
#pragma unroll
      for (int u = 0; u < 8; u += 2) {
        acc0 = Mfma<T>::run(av[u], bv[u], acc0);
        acc1 = Mfma<T>::run(av[u + 1], bv[u + 1], acc1);
      }
    }
    if (wave < 15) {
      T *dst = R4 + sl * kJgPart + tile * 256;
#pragma unroll
      for (int v = 0; v < 4; ++v) dst[Mfma<T>::row(lane, v) * 16 + r16] = acc0[v] + acc1[v];
    }
  }
  __syncthreads();
  {
    // entry (i, j) of G from the five partial sums of its block (the block above the diagonal read transposed below it)
    const int i = tid >> 5, j = tid & 31;
    const int bi2 = i >> 4, bj2 = j >> 4;
    const bool lower = bi2 > bj2;
    const int tile = lower ? 1 : bi2 + bj2;
    const int e = tile * 256 + (lower ? (j & 15) * 16 + (i & 15) : (i & 15) * 16 + (j & 15));
    G0[i * kJgLd + j] = ((R4[e] + R4[kJgPart + e]) + (R4[2 * kJgPart + e] + R4[3 * kJgPart + e])) + R4[4 * kJgPart + e];
  }
  __syncthreads();
  T *Tb[2] = {R4, R4 + kJgMat};
  T *Gb[2] = {G0, R4 + 2 * kJgMat};
  {
    const int i = tid >> 5, j = tid & 31;
    Tb[0][i * kJgLd + j] = (i == j) ? (T)1 : (T)0;
  }
  __syncthreads();

  // b rounds.  Wavefronts 0-3 (one per SIMD: the chain of dependent instructions of a round is theirs alone):
  // G <- J^T G J, thread (a, bb) the rows of pair a and the columns of pair bb; every lane works out the rotation of
  // pair bb = lane mod 16, fetches that of pair a from lane a, and the first sixteen leave (c, s) of the round in
  // LDS.  Wavefronts 4-11: T <- T J one round behind, thread (rr, bb) row rr and the columns of pair bb.  One barrier
  // per round (G and T alternate between two copies).
  const T floor2 = (T)(Eps<T>::value * Eps<T>::value * hdr->fro2);
  T *CS = R4 + 3 * kJgMat;                                     // [b rounds][16 pairs][c, s], in the fourth matrix
  float rho = 0.f;
  const int bb = tid & 15;
  auto rotate_t = [&](int r) {                                 // T <- T J_r
    const T *Ts = Tb[r & 1];
    T *Td = Tb[(r & 1) ^ 1];
    const int rr = (tid - 256) >> 4;
    const int qb = kJgB + ((bb + r) & (kJgB - 1));
    const T cb = CS[(r * 16 + bb) * 2], sb = CS[(r * 16 + bb) * 2 + 1];
    const T tp = Ts[rr * kJgLd + bb], tq = Ts[rr * kJgLd + qb];
    Td[rr * kJgLd + bb] = cb * tp - sb * tq;
    Td[rr * kJgLd + qb] = sb * tp + cb * tq;
  };
  for (int r = 0; r < b; ++r) {
    if (tid < 256) {
      const T *Gs = Gb[r & 1];
      T *Gd = Gb[(r & 1) ^ 1];
      int qb;
      T cb, sb;
      const float rel = jg_pair_params<T>(Gs, bb, r, cols_i, cols_j, tol, floor2, qb, cb, sb);
      const int a = tid >> 4;
      const int qa = kJgB + ((a + r) & (kJgB - 1));
      const T g00 = Gs[a * kJgLd + bb], g01 = Gs[a * kJgLd + qb];
      const T g10 = Gs[qa * kJgLd + bb], g11 = Gs[qa * kJgLd + qb];
      const T ca = lane_read<T>(cb, a), sa = lane_read<T>(sb, a);
      const T h00 = ca * g00 - sa * g10, h01 = ca * g01 - sa * g11;
      const T h10 = sa * g00 + ca * g10, h11 = sa * g01 + ca * g11;
      T n00 = cb * h00 - sb * h01, n01 = sb * h00 + cb * h01;
      T n10 = cb * h10 - sb * h11, n11 = sb * h10 + cb * h11;
      if (a == bb && rel > 0.f) {
        n01 = (T)0;
        n10 = (T)0;
        rho = fmaxf(rho, rel);
      }
      Gd[a * kJgLd + bb] = n00; Gd[a * kJgLd + qb] = n01;
      Gd[qa * kJgLd + bb] = n10; Gd[qa * kJgLd + qb] = n11;
      if (a == 0) {
        CS[(r * 16 + bb) * 2] = cb;
        CS[(r * 16 + bb) * 2 + 1] = sb;
      }
    } else if (tid < 768 && r > 0) {
      rotate_t(r - 1);
    }
    __syncthreads();
  }
  if (tid >= 256 && tid < 768) rotate_t(b - 1);
  if (rho > 0.f) atomicMax(&rotations, __float_as_int(rho));
  __syncthreads();
  const int rho_bits = rotations;
  if (rho_bits == 0) {                                        // nothing changed: leave M alone, no T to apply
    if (tid == 0) chg[slot * nblk + blockIdx.x] = 0;
    return;
  }
  const T *Tf = Tb[b & 1];                                    // T[k][j]
  // panel out: (P T)^T = T^T P^T in 16 x 16 blocks; wavefront w takes the output columns jb * 16 ... and the row
  // blocks rb, rb + 8, ..., two of them at a time
  {
    const int jb = wave & 1;
    T ta[kJgN / 4];
#pragma unroll
    for (int ks = 0; ks < kJgN / 4; ++ks) ta[ks] = Tf[(4 * ks + kq) * kJgLd + jb * 16 + r16];     // A[i = column][k] = T[k][column]
    const int nrb = lp / 16;
    for (int rb = wave >> 1; rb < nrb; rb += 16) {
      const int rb2 = rb + 8;
      const bool two = rb2 < nrb;
      const T *bp0 = Pc + kq * ldp + rb * 16 + r16;                                              // B[k][n = row] = P[row][k]
      const T *bp1 = Pc + kq * ldp + (two ? rb2 : rb) * 16 + r16;
      T b0[kJgN / 4], b1[kJgN / 4];
#pragma unroll
      for (int ks = 0; ks < kJgN / 4; ++ks) { b0[ks] = bp0[(4 * ks) * ldp]; b1[ks] = bp1[(4 * ks) * ldp]; }
      acc_t acc0 = (acc_t)(T)0, acc1 = (acc_t)(T)0;
#pragma unroll
      for (int ks = 0; ks < kJgN / 4; ++ks) {
        acc0 = Mfma<T>::run(ta[ks], b0[ks], acc0);
        acc1 = Mfma<T>::run(ta[ks], b1[ks], acc1);
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int c = jb * 16 + Mfma<T>::row(lane, v);
        if (live(c)) {
          T *dst = Mt + (int64_t)gcol(c) * l;
          if (rb * 16 + r16 < l) dst[rb * 16 + r16] = acc0[v];
          if (two && rb2 * 16 + r16 < l) dst[rb2 * 16 + r16] = acc1[v];
        }
      }
    }
  }
  T *Tg = Tring + ((size_t)slot * nblk + blockIdx.x) * (size_t)(4 * b * b);
  {
    // ring format: Tg[c * 2b + k] = T[k][c] over the live columns, packed (those of the first block, then the second)
    const int c = tid >> 5, k = tid & 31;
    auto unpack = [&](int x) { return x < cols_i ? x : b + (x - cols_i); };
    T val = (T)0;
    if (c < ncols && k < ncols) val = Tf[unpack(k) * kJgLd + unpack(c)];
    else if (c == k) val = (T)1;
    Tg[c * (2 * b) + k] = val;
  }
  if (tid == 0) {
    chg[slot * nblk + blockIdx.x] = 1;
    atomicMax(&hdr->counters[sweep], rho_bits);
  }
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
  // the norms go through LDS a chunk at a time (one after the other from global memory, the l comparisons of a
  // thread took 33 us at l = 576)
  __shared__ T chunk[1024];
  const T mine = j < l ? nrm[j] : (T)0;
  int rank = 0;
  for (int c0 = 0; c0 < l; c0 += 1024) {
    const int cn = (l - c0 < 1024) ? (l - c0) : 1024;
    for (int i = threadIdx.x; i < cn; i += blockDim.x) chunk[i] = nrm[c0 + i];
    __syncthreads();
    if (j < l) {
      for (int i = 0; i < cn; ++i) {
        const T o = chunk[i];
        rank += (o > mine || (o == mine && c0 + i < j)) ? 1 : 0;
      }
    }
    __syncthreads();
  }
  if (j < l) {
    rnk[j] = rank;
    sigma[rank] = mine * (T)hdr->unscale;
  }
  if (j == 0 && info != nullptr) {
    const float tol = (float)(Eps<T>::value * sqrt((T)l));
    int used = max_sweeps;
    for (int s = 1; s <= max_sweeps; ++s)
      if (jacobi_done_before(hdr->counters, s, tol)) { used = s; break; }
    atomicMax(&info->jacobi_sweeps, used);
    if (!jacobi_done_before(hdr->counters, max_sweeps, tol)) atomicMax(&info->status, (int)RSVD_ERR_NO_CONVERGENCE);
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

// Lanes per column pair of the LDS-resident kernel.
static int jacobi_group(rsvd_dtype dtype, int64_t l) {
  (void)dtype; (void)l;
  return 16;       // measured: 16 beats 8 from l = 20 to 128 (a round is one wavefront's dependent chain), 4 is slowest
}

static size_t jacobi_lds_bytes(rsvd_dtype dtype, int64_t l) {
  const size_t es = dtype_size(dtype);
  const size_t ldm = (size_t)jacobi_ldm((int)l, jacobi_group(dtype, l), (int)es);
  return align_up(2 * (size_t)l * ldm * es + (size_t)l * (es + sizeof(int)), 16);
}

int jacobi_max_lds_order(const rsvd_ctx *ctx, rsvd_dtype dtype) {
  int l = 2;
  while (l < 128 && jacobi_lds_bytes(dtype, l + 1) + 4096 <= ctx->lds_per_block) ++l;
  return l;      // 128 columns = 64 pairs x 16 lanes = the largest workgroup
}

// Largest order of a batched call: fp64 orders beyond the LDS-resident kernel keep J in global memory, up to the
// largest workgroup (64 pairs x 16 lanes).
int jacobi_max_batched_order(const rsvd_ctx *ctx, rsvd_dtype dtype) {
  return dtype == RSVD_F64 ? 128 : jacobi_max_lds_order(ctx, dtype);
}
static size_t jacobi_jglobal_bytes(int64_t l) {
  return (size_t)l * (size_t)jacobi_ldm((int)l, 16, 8) * 8;
}

// Units (8 bytes) per lane for order l: ceil(l / V / 32), rounded up to an instantiated value.
static int jb_units_per_lane(rsvd_dtype dtype, int64_t l) {
  const int v = 8 / (int)dtype_size(dtype);
  const int need = (int)ceil_div(ceil_div(l, v), 32);
  static const int avail[] = {2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 14, 16, 18, 20, 24};
  for (int a : avail)
    if (a >= need) return a;
  return 0;
}

// block width for the panel kernel: b padded columns plus the 2b x 2b T must fit in LDS
static int jb_block_width(const rsvd_ctx *ctx, rsvd_dtype dtype, int64_t l) {
  const size_t es = dtype_size(dtype);
  const int nv = jb_units_per_lane(dtype, l);
  if (nv == 0) return 0;
  const size_t ldp = (size_t)32 * nv * (8 / es) + 2;
  // Measured from l = 130 to 576 in both precisions: 16 beats 24 and 32 (a round is bound by instruction issue,
  // so fewer wavefronts per SIMD make it shorter, which outweighs the larger number of launches), 8 is slower.
  for (int b = 16; b >= 8; b -= 8) {
    const size_t need = ((size_t)b * ldp + (size_t)(2 * b) * (2 * b + 2)) * es + 1024;   // one block of columns + T
    if (need <= ctx->lds_per_block) return b;
  }
  return 0;
}

// Scratch of the block path: header, Mt, Jt, norms, ranks.
size_t jacobi_scratch_bytes(const rsvd_ctx *ctx, rsvd_dtype dtype, int64_t l) {
  if (l <= jacobi_max_lds_order(ctx, dtype)) return 0;
  if (jb_block_width(ctx, dtype, l) == 0) return 0;          // unsupported order
  const size_t es = dtype_size(dtype);
  const size_t b = (size_t)jb_block_width(ctx, dtype, l), nblk = ceil_div((size_t)l, b);
  return align_up(sizeof(JbHeader), 256) + 2 * align_up((size_t)l * l * es, 256) + align_up((size_t)l * es, 256) +
         align_up((size_t)l * sizeof(int), 256) + align_up(2 * nblk * 4 * b * b * es, 256) +
         align_up(2 * nblk * sizeof(int), 256);
}

template <typename T>
static hipError_t jacobi_block_launch(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype dtype, int l, const double *M,
                                      T *sigma, T *X, T *W, DevInfo *info, char *scratch, int rows) {
  const int b = jb_block_width(ctx, dtype, l);
  if (b == 0) return hipErrorNotSupported;
  const size_t es = sizeof(T);
  JbHeader *hdr = reinterpret_cast<JbHeader *>(scratch);
  char *p = scratch + align_up(sizeof(JbHeader), 256);
  T *Mt = reinterpret_cast<T *>(p); p += align_up((size_t)l * l * es, 256);
  T *Jt = reinterpret_cast<T *>(p); p += align_up((size_t)l * l * es, 256);
  T *nrm = reinterpret_cast<T *>(p); p += align_up((size_t)l * es, 256);
  int *rnk = reinterpret_cast<int *>(p); p += align_up((size_t)l * sizeof(int), 256);
  const int nblk = (l + b - 1) / b;
  T *Tring = reinterpret_cast<T *>(p); p += align_up((size_t)2 * nblk * 4 * b * b * es, 256);   // [2][nblk][2b][2b]
  int *chg = reinterpret_cast<int *>(p);                                                        // [2][nblk]
  const int nblk2 = nblk + (nblk & 1);
  const int nv = jb_units_per_lane(dtype, l);
  const size_t ldp = (size_t)32 * nv * (8 / es) + 2;
  const size_t lds_rot = ((size_t)b * ldp + (size_t)(2 * b) * (2 * b + 2)) * es;
  const size_t lds_j = ((size_t)(2 * b) * (kJbRowChunk + 8) + (size_t)(2 * b) * (2 * b + 2)) * es;   // jb_apply_t
  const size_t lds = lds_rot > lds_j ? lds_rot : lds_j;
  const int chunks = (l + kJbRowChunk - 1) / kJbRowChunk;
  // cross launches go through the Gram matrix of the block pair when its panel of 2b columns fits in LDS
  const bool gram_cross = b == kJgB && jg_lds_bytes<T>(l) + 1024 <= ctx->lds_per_block;
  const size_t lds_gram = jg_lds_bytes<T>(l) > lds_j ? jg_lds_bytes<T>(l) : lds_j;
  ProfScope ps(ctx, s, PK_JACOBI);
  hipLaunchKernelGGL(jb_fro_kernel, dim3(kJbFroParts), dim3(256), 0, s, M, l, hdr);
  {
    int64_t blocks = ((int64_t)l * l + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL((jb_init_kernel<T>), dim3((unsigned)blocks), dim3(256), 0, s, M, l, Mt, Jt, hdr, rows);
  }
#define RSVD_JB_CASE(NVV)                                                                                        \
  case NVV: {                                                                                                    \
    int slot = 0, pp = -1, pr = 0, psw = 0, pwgs = 0;          /* the launch before: phase, round, sweep, pairs */ \
    auto go = [&](int phase, int round, int sweep, int wgs) {                                                    \
      if (phase == 1 && wgs > 0 && gram_cross)                                                                   \
        hipLaunchKernelGGL((jb_cross_kernel<T>), dim3(wgs + pwgs * chunks), dim3(1024), lds_gram, s, Mt, Jt, l,  \
                           nblk, round, sweep, wgs, pp, pr, psw, Tring, chg, slot, hdr);                         \
      else                                                                                                       \
        hipLaunchKernelGGL((jb_panel_kernel<T, NVV>), dim3(wgs + pwgs * chunks), dim3(1024), lds, s, Mt, Jt, l,  \
                           b, nblk, phase, round, sweep, wgs, pp, pr, psw, Tring, chg, slot, hdr);               \
      pp = phase; pr = round; psw = sweep; pwgs = wgs; slot ^= 1;                                                \
    };                                                                                                           \
    for (int sweep = 0; sweep < kJbMaxSweeps; ++sweep) {                                                         \
      go(0, 0, sweep, nblk);                                                                                     \
      for (int round = 0; round < nblk2 - 1; ++round) go(1, round, sweep, nblk2 / 2);                            \
    }                                                                                                            \
    go(0, 0, kJbMaxSweeps, 0);                                 /* applies the T of the last round */            \
  } break
  switch (nv) {
    RSVD_JB_CASE(2); RSVD_JB_CASE(3); RSVD_JB_CASE(4); RSVD_JB_CASE(5); RSVD_JB_CASE(6); RSVD_JB_CASE(7);
    RSVD_JB_CASE(8); RSVD_JB_CASE(9); RSVD_JB_CASE(10); RSVD_JB_CASE(12); RSVD_JB_CASE(14); RSVD_JB_CASE(16);
    RSVD_JB_CASE(18); RSVD_JB_CASE(20); RSVD_JB_CASE(24);
    default: return hipErrorNotSupported;
  }
#undef RSVD_JB_CASE
  hipLaunchKernelGGL((jb_norms_kernel<T>), dim3((l + 3) / 4), dim3(256), 0, s, Mt, l, nrm);
  hipLaunchKernelGGL((jb_rank_kernel<T>), dim3((l + 255) / 256), dim3(256), 0, s, nrm, l, rnk, sigma, hdr,
                     kJbMaxSweeps, info);
  hipLaunchKernelGGL((jb_scatter_kernel<T>), dim3(256), dim3(256), 0, s, Mt, Jt, l, nrm, rnk, hdr, X, W);
  return hipGetLastError();
}

template <typename T, typename TIn, int RPL, int G>
static hipError_t launch_lds(hipStream_t s, int nt, size_t lds, const void *M, int l, void *sigma, void *X, void *W,
                             DevInfo *info, int batch, int64_t stride, int rows) {
  hipLaunchKernelGGL((jacobi_lds_kernel<T, TIn, RPL, G>), dim3(batch), dim3(nt), lds, s, (const TIn *)M, l,
                     (T *)sigma, (T *)X, (T *)W, info, stride, rows, (T *)nullptr);
  return hipGetLastError();
}
// fp64 orders 97 .. 128: M in LDS, J in global memory
template <int RPL>
static hipError_t launch_lds_jg(hipStream_t s, int nt, size_t lds, const void *M, int l, void *sigma, void *X, void *W,
                                DevInfo *info, int batch, int64_t stride, int rows, void *Jglobal) {
  hipLaunchKernelGGL((jacobi_lds_kernel<double, double, RPL, 16, true>), dim3(batch), dim3(nt), lds, s,
                     (const double *)M, l, (double *)sigma, (double *)X, (double *)W, info, stride, rows,
                     (double *)Jglobal);
  return hipGetLastError();
}

// rows per lane = padded rows / G
template <typename T, typename TIn>
static hipError_t launch_lds_g(hipStream_t s, int nt, int G, int rpl, size_t lds, const void *M, int l, void *sigma,
                               void *X, void *W, DevInfo *info, int batch, int64_t stride, int rows) {
  if (G == 16) {
    // fp32 rows come in pairs (8-byte units), fp64 rows singly
    if constexpr (sizeof(T) == 8) {
      switch (rpl) {
        case 1: return launch_lds<T, TIn, 1, 16>(s, nt, lds, M, l, sigma, X, W, info, batch, stride, rows);
        case 3: return launch_lds<T, TIn, 3, 16>(s, nt, lds, M, l, sigma, X, W, info, batch, stride, rows);
        case 5: return launch_lds<T, TIn, 5, 16>(s, nt, lds, M, l, sigma, X, W, info, batch, stride, rows);
        default: break;
      }
    }
    switch (rpl) {
      case 2: return launch_lds<T, TIn, 2, 16>(s, nt, lds, M, l, sigma, X, W, info, batch, stride, rows);
      case 4: return launch_lds<T, TIn, 4, 16>(s, nt, lds, M, l, sigma, X, W, info, batch, stride, rows);
      case 6: return launch_lds<T, TIn, 6, 16>(s, nt, lds, M, l, sigma, X, W, info, batch, stride, rows);
      case 8: return launch_lds<T, TIn, 8, 16>(s, nt, lds, M, l, sigma, X, W, info, batch, stride, rows);
      default: return hipErrorNotSupported;
    }
  }
  return hipErrorNotSupported;
}

// The kernels of this file are launched with up to 156 KB of dynamic LDS: the limit is raised here, once per
// context (with its device current), for every instantiation the dispatch above can reach.
template <typename T, typename TIn, int RPL>
static void raise_lds_limit_lds(hipError_t &e) {
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&jacobi_lds_kernel<T, TIn, RPL, 16>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 4096);
}
template <int RPL>
static void raise_lds_limit_jg(hipError_t &e) {
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&jacobi_lds_kernel<double, double, RPL, 16, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 4096);
}
template <typename T, int NV>
static void raise_lds_limit_panel(hipError_t &e) {
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&jb_panel_kernel<T, NV>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 4096);
}
template <typename T>
static void raise_lds_limit_panels(hipError_t &e) {
  raise_lds_limit_panel<T, 2>(e); raise_lds_limit_panel<T, 3>(e); raise_lds_limit_panel<T, 4>(e);
  raise_lds_limit_panel<T, 5>(e); raise_lds_limit_panel<T, 6>(e); raise_lds_limit_panel<T, 7>(e);
  raise_lds_limit_panel<T, 8>(e); raise_lds_limit_panel<T, 9>(e); raise_lds_limit_panel<T, 10>(e);
  raise_lds_limit_panel<T, 12>(e); raise_lds_limit_panel<T, 14>(e); raise_lds_limit_panel<T, 16>(e);
  raise_lds_limit_panel<T, 18>(e); raise_lds_limit_panel<T, 20>(e); raise_lds_limit_panel<T, 24>(e);
}

hipError_t jacobi_init_device(rsvd_ctx *ctx) {
  (void)ctx;
  hipError_t e = hipSuccess;
  raise_lds_limit_lds<float, double, 2>(e); raise_lds_limit_lds<float, double, 4>(e);
  raise_lds_limit_lds<float, double, 6>(e); raise_lds_limit_lds<float, double, 8>(e);
  raise_lds_limit_lds<float, float, 2>(e); raise_lds_limit_lds<float, float, 4>(e);
  raise_lds_limit_lds<float, float, 6>(e); raise_lds_limit_lds<float, float, 8>(e);
  raise_lds_limit_lds<double, double, 1>(e); raise_lds_limit_lds<double, double, 2>(e);
  raise_lds_limit_lds<double, double, 3>(e); raise_lds_limit_lds<double, double, 4>(e);
  raise_lds_limit_lds<double, double, 5>(e); raise_lds_limit_lds<double, double, 6>(e);
  raise_lds_limit_lds<double, double, 8>(e);
  raise_lds_limit_jg<7>(e);
  raise_lds_limit_jg<8>(e);
  raise_lds_limit_panels<float>(e);
  raise_lds_limit_panels<double>(e);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&jb_cross_kernel<float>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 4096);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&jb_cross_kernel<double>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 4096);
  return e;
}

hipError_t jacobi_launch(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype dtype, int64_t l, const void *M,
                         int m_is_f64, void *sigma, void *X, void *W, DevInfo *info, void *scratch,
                         size_t scratch_bytes, int batch, int64_t stride, int rows) {
  if (batch < 1 || batch > 65535) return hipErrorInvalidValue;
  if (l > jacobi_max_lds_order(ctx, dtype)) {
    if (batch != 1) {
      // the block path is not batched: fp64 orders up to 128 take the one-workgroup kernel with J in global memory
      // (the block path's scratch, which every problem of the batch has, is larger than one J)
      if (dtype != RSVD_F64 || l > jacobi_max_batched_order(ctx, dtype) || !m_is_f64 || scratch == nullptr ||
          scratch_bytes < jacobi_jglobal_bytes(l))
        return hipErrorNotSupported;
      const int ldm = jacobi_ldm((int)l, 16, 8);
      const size_t lds = align_up((size_t)l * ldm * 8 + (size_t)l * (8 + sizeof(int)), 16);
      const int nt = (int)align_up((size_t)((l + 1) / 2) * 16, 64);
      ProfScope ps(ctx, s, PK_JACOBI);
      if (jacobi_rows_padded((int)l, 16, 8) / 16 == 7)
        return launch_lds_jg<7>(s, nt, lds, M, (int)l, sigma, X, W, info, batch, stride, rows, scratch);
      return launch_lds_jg<8>(s, nt, lds, M, (int)l, sigma, X, W, info, batch, stride, rows, scratch);
    }
    // block path: needs the fp64 input (the triangular factor) and its scratch
    const size_t need = jacobi_scratch_bytes(ctx, dtype, l);
    if (need == 0 || scratch == nullptr || scratch_bytes < need || !m_is_f64) return hipErrorNotSupported;
    if (dtype == RSVD_F32)
      return jacobi_block_launch<float>(ctx, s, dtype, (int)l, (const double *)M, (float *)sigma, (float *)X,
                                        (float *)W, info, (char *)scratch, rows);
    return jacobi_block_launch<double>(ctx, s, dtype, (int)l, (const double *)M, (double *)sigma, (double *)X,
                                       (double *)W, info, (char *)scratch, rows);
  }
  // one G-lane group per column pair of a round, all pairs of a round at once
  const int npairs = (int)((l + 1) / 2);
  const int G = jacobi_group(dtype, l);
  int nt = (int)align_up((size_t)npairs * G, 64);
  if (nt > 64 * G) nt = 64 * G;
  const int g = jacobi_rows_padded((int)l, G, (int)dtype_size(dtype)) / G;          // rows per lane
  const size_t lds = jacobi_lds_bytes(dtype, l);
  ProfScope ps(ctx, s, PK_JACOBI);
  if (dtype == RSVD_F32) {
    if (m_is_f64) return launch_lds_g<float, double>(s, nt, G, g, lds, M, (int)l, sigma, X, W, info, batch, stride, rows);
    return launch_lds_g<float, float>(s, nt, G, g, lds, M, (int)l, sigma, X, W, info, batch, stride, rows);
  }
  return launch_lds_g<double, double>(s, nt, G, g, lds, M, (int)l, sigma, X, W, info, batch, stride, rows);
}

}  // namespace rsvd
