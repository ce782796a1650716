// MFMA GEMM for the tall-skinny / short-wide products of Algorithm 1
// (steps 2, 4 and 6: products of A, A^T and Q with n x l, m x l and l x k
// blocks; also the Gram matrices and triangular applies of step 3).
//
// One template covers every product:  C = alpha * op(A) * B + beta * C  with
//   op(A) = A   (row-major M x K)  : tiles of A are staged in LDS as [row][k]
//   op(A) = A^T (A stored K x M)   : tiles are staged as [k][row]
// B is always K x N row-major (the skinny operand), staged as [k][col].
// A 256-thread workgroup (4 wavefronts arranged WGM x WGN) owns a BM x BN tile of
// C; each wavefront owns TM x TN blocks of 16 x 16 and issues
// v_mfma_{f32,f64}_16x16x4 on fragments read from LDS.  The K range can be split
// over gridDim.z; partial tiles then go to a scratch buffer and a second kernel
// adds them in a fixed order, so results do not depend on scheduling.
//
// Included by gemm_f32.hip, gemm_f64.hip and gemm_f32acc64.hip, one per
// (input type, accumulator type) pair.
#pragma once

#include "common.hpp"
#include "mfma.hpp"
#include "philox_dev.hpp"

namespace rsvd {

struct GemmParams {
  int64_t M, N, K;
  const void *A; int64_t lda;
  const void *B; int64_t ldb;
  void *C; int64_t ldc;
  void *partial;            // [splits][M][N] accumulator-typed, used when splits > 1
  int64_t k_per_split;
  int splits;
  int tiles_n, tiles_m;     // grid shape in tiles; the launch is one-dimensional
  int upper_bm, upper_bn;   // > 0: symmetric result, tiles (of this size) strictly below the diagonal are skipped
  int b_upper;              // != 0: B is upper triangular (row k is zero before column k): a column tile ends its k range early
  int trans_c;
  double alpha, beta;
  const double *a_shift;    // non-NULL: op(A) is built from A[i][j] - a_shift[j] (one value per column of A)
  const int *dead;
  uint64_t seed; uint32_t refill_stream; double refill_scale; int64_t refill_ld;
  // batched launch (blockIdx.y = problem): byte strides of the pointers above, seed step
  int64_t stride_a, stride_b, stride_c, stride_partial, stride_dead;
  uint64_t seed_step;
  // device-side switches (ints in device memory, one per problem, stride_flag bytes apart; may be NULL):
  //   *skip_flag != 0: the launch does nothing;  *alt_flag != 0: B_alt takes the place of B
  const int *skip_flag; const int *alt_flag; const void *B_alt; int64_t stride_flag;
  int skip_now;             // filled in on the device
  int reduce_groups;        // split-K reduction: threads per output element (1, 2, 4 or 8)
};

// The parameters of problem blockIdx.y of a batched launch.
__device__ __forceinline__ GemmParams select_problem(const GemmParams &P0) {
  GemmParams P = P0;
  const int64_t b = (int64_t)blockIdx.y;
  if (b != 0) {
    P.A = (const char *)P.A + b * P.stride_a;
    P.B = (const char *)P.B + b * P.stride_b;
    P.C = (char *)P.C + b * P.stride_c;
    if (P.partial != nullptr) P.partial = (char *)P.partial + b * P.stride_partial;
    if (P.dead != nullptr) P.dead = (const int *)((const char *)P.dead + b * P.stride_dead);
    P.seed += (uint64_t)b * P.seed_step;
  }
  P.skip_now = 0;
  if (P.skip_flag != nullptr) P.skip_now = *(const int *)((const char *)P.skip_flag + b * P.stride_flag);
  if (P.alt_flag != nullptr && *(const int *)((const char *)P.alt_flag + b * P.stride_flag) != 0)
    P.B = (const char *)P.B_alt + b * P.stride_b;
  return P;
}

// Final store of one element of C, shared by the GEMM and the split-K reduction.
template <typename TOut, typename TAcc, bool F32STREAM>
__device__ __forceinline__ void store_result(const GemmParams &P, int64_t row, int64_t col, TAcc acc) {
  TOut *C = (TOut *)P.C;
  double v = P.alpha * (double)acc;
  if (P.dead != nullptr && P.dead[col] != 0) {
    v = P.refill_scale *
        philox_normal_at<F32STREAM>((uint64_t)(row * P.refill_ld + col), P.refill_stream, P.seed);
  }
  if (P.trans_c) {
    C[col * P.ldc + row] = (TOut)v;
  } else {
    TOut *p = C + row * P.ldc + col;
    if (P.beta != 0.0) v += P.beta * (double)(*p);
    *p = (TOut)v;
  }
}

// LDS padding: k-major tiles ([k][x], lanes read 16 consecutive x for 4 consecutive k)
// want a row stride that is not a multiple of 32 words.
__host__ __device__ constexpr int pad_kmajor(int x) { return (x % 32 == 0) ? 16 : 0; }

// SHIFT: the tile is a piece of a matrix whose columns carry an offset that is taken away on the way
// to LDS (in fp64, rounded once): element (r, c) becomes x - shift[c].  The subtraction waits for
// store(), so that the loads of the next tile stay in flight behind the matrix instructions.
// (Tried: the offset as a pair of floats, and the subtraction placed behind the matrix instructions
// of the tile before; neither was faster.)
template <typename TIn, int ROWS, int COLS, int VEC, bool SHIFT = false>
struct TileStage {
  static constexpr int SLOTS_PER_ROW = COLS / VEC;
  static constexpr int SLOTS = ROWS * SLOTS_PER_ROW;
  static constexpr int ITERS = (SLOTS + 255) / 256;
  static_assert(!SHIFT || 256 % SLOTS_PER_ROW == 0, "a thread must stay in one column group");
  TIn regs[ITERS][VEC];
  double sh[SHIFT ? VEC : 1];
  unsigned valid;            // SHIFT: bit it = the slot of iteration it holds data (padding stays zero)

  // rows_left / cols_left: extent of valid data from the tile origin (may exceed the tile).
  // shift: the offsets of the tile's columns (SHIFT only); NULL keeps those of the load before.
  // (Predicated loads behind a branch measured faster than unconditional loads from a clamped
  // address followed by a select.)
  __device__ __forceinline__ void load(const TIn *__restrict__ origin, int64_t ld, int64_t rows_left,
                                       int64_t cols_left, int tid, const double *__restrict__ shift = nullptr) {
    if (SHIFT) {
      valid = 0u;
      if (shift != nullptr) {
        const int c = (tid % SLOTS_PER_ROW) * VEC;
#pragma unroll
        for (int e = 0; e < VEC; ++e) sh[e] = (c + e < cols_left) ? shift[c + e] : 0.0;
      }
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const int idx = tid + it * 256;
      const int r = idx / SLOTS_PER_ROW;
      const int c = (idx - r * SLOTS_PER_ROW) * VEC;
      const bool ok = (ITERS * 256 == SLOTS || idx < SLOTS) && r < rows_left && c < cols_left;
      if (SHIFT && ok) valid |= 1u << it;
      if (VEC == 1) {
        regs[it][0] = ok ? origin[(int64_t)r * ld + c] : (TIn)0;
      } else {
        typedef TIn vec_t __attribute__((ext_vector_type(VEC)));
        vec_t v = (vec_t)(TIn)0;
        if (ok) v = *reinterpret_cast<const vec_t *>(origin + (int64_t)r * ld + c);
#pragma unroll
        for (int e = 0; e < VEC; ++e) regs[it][e] = v[e];
      }
    }
  }
  __device__ __forceinline__ void store(TIn *lds, int stride, int tid) const {
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const int idx = tid + it * 256;
      if (ITERS * 256 == SLOTS || idx < SLOTS) {
        const int r = idx / SLOTS_PER_ROW;
        const int c = (idx - r * SLOTS_PER_ROW) * VEC;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          TIn x = regs[it][e];
          if (SHIFT) x = ((valid >> it) & 1u) ? (TIn)((double)x - sh[e]) : (TIn)0;
          lds[r * stride + c + e] = x;
        }
      }
    }
  }
};

// Epilogues (EPI):
//   0  the kernel can only store its tile as it is (or as a split-K partial);
//   1  the full epilogue (scaling, accumulation, transposed store, replacement columns);
//   2  C = alpha * acc + beta * C only, with all of a thread's old values of C loaded before the
//      first store (element by element the loads would queue behind the stores, one memory
//      round trip each);
//   3  as 0, with the column offsets P.a_shift taken away from A while its tiles are staged
//      (the centred products: A - 1 mu^T is never formed, and no cancellation happens after
//      the fact as it would with a rank-one correction of the product).
// Separate instantiations: the full epilogue carries the Philox and Box-Muller code and more registers,
// which the products with A never need.
template <typename TIn, typename TAcc, typename TOut, bool TA, int BM, int BN, int WGM, int WGN, int VEC, int EPI,
          int BK = 32>
__global__ __launch_bounds__(256) void gemm_kernel(const GemmParams P0) {
  const GemmParams P = select_problem(P0);
  if (P.skip_now) return;
  static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
  constexpr int WM = BM / WGM, WN = BN / WGN;
  static_assert(WM % 16 == 0 && WN % 16 == 0, "wave tile must be made of 16x16 blocks");
  constexpr int TM = WM / 16, TN = WN / 16;
  // LDS strides (elements)
  constexpr int SA = TA ? (BM + pad_kmajor(BM)) : (BK + (sizeof(TIn) == 4 ? 4 : 2));
  constexpr int SB = BN + pad_kmajor(BN);
  constexpr int A_ROWS = TA ? BK : BM, A_COLS = TA ? BM : BK;
  __shared__ TIn As[A_ROWS * SA];
  __shared__ TIn Bs[BK * SB];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;
  const int r16 = lane & 15, kq = lane >> 4;

  // Workgroups are handed to the 8 XCDs round-robin by launch index, and each XCD has
  // its own L2.  Renumber so that one XCD receives a contiguous run of tile indices:
  // the column tiles of one row tile (which all read the same rows of A) then share an L2.
  const int total = (int)gridDim.x;
  const int pid = (int)blockIdx.x;
  const int per_xcd = (total + 7) >> 3;
  const int tall = (total & 7) ? (total & 7) : 8;        // XCDs that receive per_xcd workgroups
  const int xcd = pid & 7, local = pid >> 3;
  const int tile = (xcd < tall) ? xcd * per_xcd + local
                                : tall * per_xcd + (xcd - tall) * (per_xcd - 1) + local;
  const int tile_n = tile % P.tiles_n;
  const int tile_m = (tile / P.tiles_n) % P.tiles_m;
  const int split = tile / (P.tiles_n * P.tiles_m);
  const int64_t m0 = (int64_t)tile_m * BM;
  const int64_t n0 = (int64_t)tile_n * BN;
  if (P.upper_bm > 0 && n0 + BN <= m0) return;       // symmetric result: this tile mirrors one that is computed
  const int64_t k_begin = (int64_t)split * P.k_per_split;
  int64_t k_end = (k_begin + P.k_per_split < P.K) ? (k_begin + P.k_per_split) : P.K;
  if (P.b_upper != 0 && n0 + BN < k_end) k_end = n0 + BN;      // rows of B from n0 + BN on are zero in these columns

  const TIn *A = (const TIn *)P.A;
  const TIn *B = (const TIn *)P.B;

  typedef typename Mfma<TAcc>::vec acc_t;
  acc_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = (acc_t)(TAcc)0;

  constexpr bool CENTER = (EPI == 3);
  TileStage<TIn, A_ROWS, A_COLS, VEC, CENTER> sa;
  TileStage<TIn, BK, BN, VEC> sb;

  auto load_tiles = [&](int64_t k0) {
    // columns of A: the rows of op(A) = A^T (the same for every k-tile), the k index otherwise
    if (TA) sa.load(A + k0 * P.lda + m0, P.lda, k_end - k0, P.M - m0, tid,
                    (CENTER && k0 == k_begin) ? P.a_shift + m0 : nullptr);
    else    sa.load(A + m0 * P.lda + k0, P.lda, P.M - m0, k_end - k0, tid, CENTER ? P.a_shift + k0 : nullptr);
    sb.load(B + k0 * P.ldb + n0, P.ldb, k_end - k0, P.N - n0, tid);
  };

  if (k_begin < k_end) load_tiles(k_begin);
  for (int64_t k0 = k_begin; k0 < k_end; k0 += BK) {
    sa.store(As, SA, tid);
    sb.store(Bs, SB, tid);
    __syncthreads();
    if (k0 + BK < k_end) load_tiles(k0 + BK);
#pragma unroll
    for (int kk = 0; kk < BK; kk += 4) {
      TAcc af[TM], bf[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int row = wm0 + i * 16 + r16;
        af[i] = (TAcc)(TA ? As[(kk + kq) * SA + row] : As[row * SA + kk + kq]);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) bf[j] = (TAcc)Bs[(kk + kq) * SB + wn0 + j * 16 + r16];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = Mfma<TAcc>::run(af[i], bf[j], acc[i][j]);
    }
    __syncthreads();
  }

  // epilogue
  if (EPI == 0 || EPI == 3 || P.splits > 1) {
    TOut *Cp = (TOut *)P.C;
    TAcc *Pp = (TAcc *)P.partial + (int64_t)split * P.M * P.N;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int64_t row = m0 + wm0 + i * 16 + Mfma<TAcc>::row(lane, v);
          const int64_t col = n0 + wn0 + j * 16 + r16;
          if (row < P.M && col < P.N) {
            if (P.splits > 1) Pp[row * P.N + col] = acc[i][j][v];
            else Cp[row * P.ldc + col] = (TOut)acc[i][j][v];
          }
        }
    return;
  }
  if (EPI == 1) {
    // Replacement columns are rare and do not depend on the accumulators: the flags of this lane's TN
    // columns are read once, the ordinary elements are stored on a short path, and the replacement
    // values follow in a rolled loop, so that the generator is in the code once (inlined per element
    // it made the kernel half again as slow, replacement or not).
    unsigned dead_cols = 0u;
    if (P.dead != nullptr) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int64_t col = n0 + wn0 + j * 16 + r16;
        if (col < P.N && P.dead[col] != 0) dead_cols |= 1u << j;
      }
    }
    TOut *Cp = (TOut *)P.C;
    const TAcc alpha = (TAcc)P.alpha, beta = (TAcc)P.beta;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int64_t row = m0 + wm0 + i * 16 + Mfma<TAcc>::row(lane, v);
          const int64_t col = n0 + wn0 + j * 16 + r16;
          if (row < P.M && col < P.N && !((dead_cols >> j) & 1u)) {
            if (P.trans_c) {
              Cp[col * P.ldc + row] = (TOut)(alpha * acc[i][j][v]);
            } else {
              TOut *dst = Cp + row * P.ldc + col;
              TAcc val = alpha * acc[i][j][v];
              if (beta != (TAcc)0) val += beta * (TAcc)(*dst);
              *dst = (TOut)val;
            }
          }
        }
    if (dead_cols != 0u) {
#pragma unroll 1
      for (int e = 0; e < TM * TN * 4; ++e) {
        const int v = e & 3, j = (e >> 2) % TN, i = (e >> 2) / TN;
        if (!((dead_cols >> j) & 1u)) continue;
        const int64_t row = m0 + wm0 + i * 16 + Mfma<TAcc>::row(lane, v);
        const int64_t col = n0 + wn0 + j * 16 + r16;
        if (row < P.M && col < P.N) store_result<TOut, TAcc, sizeof(TIn) == 4>(P, row, col, (TAcc)0);
      }
    }
  }
  if (EPI == 2) {
    TOut *Cp = (TOut *)P.C;
    const TAcc alpha = (TAcc)P.alpha, beta = (TAcc)P.beta;
    if (beta != (TAcc)0) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int64_t row = m0 + wm0 + i * 16 + Mfma<TAcc>::row(lane, v);
            const int64_t col = n0 + wn0 + j * 16 + r16;
            const TAcc old = (row < P.M && col < P.N) ? (TAcc)Cp[row * P.ldc + col] : (TAcc)0;
            acc[i][j][v] = alpha * acc[i][j][v] + beta * old;
          }
    } else {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] *= alpha;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int64_t row = m0 + wm0 + i * 16 + Mfma<TAcc>::row(lane, v);
          const int64_t col = n0 + wn0 + j * 16 + r16;
          if (row < P.M && col < P.N) Cp[row * P.ldc + col] = (TOut)acc[i][j][v];
        }
  }
}

// Sum of the split-K partials.  SG (1, 2, 4 or 8, P.reduce_groups) threads share one element: thread
// group g adds the partials g, g + SG, g + 2 SG, ... (eight loads in flight each), and the SG sums are
// added in the order g = 0, 1, ... through LDS - a fixed order for a given launch, so the result stays
// bitwise reproducible.  A small output with many partials (a Gram matrix of a tall panel) otherwise
// has too few threads to keep the memory system busy.
template <typename TIn, typename TAcc, typename TOut>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const GemmParams P0) {
  const GemmParams P = select_problem(P0);
  if (P.skip_now) return;
  __shared__ TAcc part[256];
  const int64_t total = P.M * P.N;
  const int SG = P.reduce_groups;
  const int EB = 256 / SG;                       // elements per workgroup and pass
  const int g = (int)threadIdx.x / EB, el = (int)threadIdx.x - g * EB;
  for (int64_t base = (int64_t)blockIdx.x * EB; base < total; base += (int64_t)gridDim.x * EB) {
    const int64_t e = base + el;
    const int64_t row = e / P.N;
    const int64_t col = e - row * P.N;
    const bool live = e < total &&
                      !(P.upper_bm > 0 && (col / P.upper_bn + 1) * P.upper_bn <= (row / P.upper_bm) * P.upper_bm);
    TAcc sum = (TAcc)0;
    if (live) {
      const TAcc *p = (const TAcc *)P.partial + e;
      int sp = g;
      for (; sp + 7 * SG < P.splits; sp += 8 * SG) {
        TAcc v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[(int64_t)(sp + u * SG) * total];
#pragma unroll
        for (int u = 0; u < 8; ++u) sum += v[u];
      }
      for (; sp < P.splits; sp += SG) sum += p[(int64_t)sp * total];
    }
    if (SG > 1) {
      part[threadIdx.x] = sum;
      __syncthreads();
      if (g == 0) {
        for (int h = 1; h < SG; ++h) sum += part[h * EB + el];
      }
      __syncthreads();
    }
    if (live && g == 0) store_result<TOut, TAcc, sizeof(TIn) == 4>(P, row, col, sum);
  }
}

// Plain sum of the partials (no scaling, no replacement columns, no transposition, full matrix), sixteen bytes
// of accumulator type per thread: the reduction of the products with A, which is pure memory traffic.
template <typename TAcc, typename TOut>
__global__ __launch_bounds__(256) void splitk_reduce_plain_kernel(const GemmParams P0) {
  const GemmParams P = select_problem(P0);
  if (P.skip_now) return;
  constexpr int V = 16 / sizeof(TAcc);
  static_assert(sizeof(TAcc) == sizeof(TOut), "same width in and out");
  typedef TAcc vacc __attribute__((ext_vector_type(V)));
  typedef TOut vout __attribute__((ext_vector_type(V)));
  const int64_t total = P.M * P.N, groups = total / V;
  for (int64_t gi = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; gi < groups; gi += (int64_t)gridDim.x * blockDim.x) {
    const int64_t e = gi * V;
    const int64_t row = e / P.N, col = e - row * P.N;
    const vacc *p = reinterpret_cast<const vacc *>((const TAcc *)P.partial + e);
    const int64_t step = total / V;
    vacc sum = (vacc)(TAcc)0;
    int sp = 0;
    for (; sp + 4 <= P.splits; sp += 4) {
      vacc v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = p[(int64_t)(sp + u) * step];
#pragma unroll
      for (int u = 0; u < 4; ++u) sum += v[u];
    }
    for (; sp < P.splits; ++sp) sum += p[(int64_t)sp * step];
    vout o;
#pragma unroll
    for (int u = 0; u < V; ++u) o[u] = (TOut)sum[u];
    *reinterpret_cast<vout *>((TOut *)P.C + row * P.ldc + col) = o;
  }
}

// ---------------------------------------------------------------- host side

struct TileChoice {
  int bm, bn;   // workgroup tile
};

// Tile shapes instantiated below (see the dispatch switch).
inline TileChoice choose_tile(int64_t M, int64_t N, int64_t K, size_t acc_size, bool trans_a, bool upper = false) {
  TileChoice t;
  if (N <= 128) {
    t.bm = 64;
    t.bn = (int)(ceil_div(N, 16) * 16);
    // symmetric result wider than 96: two column tiles, so that the tile under the diagonal can be skipped
    if (upper && N > 96) t.bn = 64;
  } else if (acc_size == 8) {
    // fp64 accumulators: the 64-row tile with one wavefront per 16 rows keeps the register
    // count low enough for two workgroups per CU
    t.bm = 64;
    const int64_t pad64 = ceil_div(N, 64) * 64 - N, pad96 = ceil_div(N, 96) * 96 - N;
    const int64_t pad128 = ceil_div(N, 128) * 128 - N;
    t.bn = 64;
    if (pad96 <= pad64) t.bn = 96;
    if (pad128 < pad64 && pad128 < pad96) t.bn = 128;
    if (trans_a && t.bn == 96) t.bm = 128;      // measured: 128 x 96 is faster for A^T X, 64 x 96 for A X
    // a short product with a handful of tiles (the panel and trailing updates of the blocked Cholesky factorisation:
    // K = 96, 5 to 20 tiles for 256 CUs) is bound by the matrix instructions of one workgroup: smaller tiles, more
    // workgroups side by side
    if (K <= 256 && ceil_div(M, t.bm) * ceil_div(N, t.bn) <= 32) { t.bm = 64; t.bn = 64; }
  } else {
    // wide outputs: 128-row tiles, column tile with the least padding.  For op(A) = A and
    // enough tiles to fill the chip twice the 192-wide tile wins on a tie (fewer LDS fragment
    // reads per matrix instruction); it measured slower for op(A) = A^T, for small grids and for
    // the short-K triangular applies.
    t.bm = 128;
    const int64_t pad96 = ceil_div(N, 96) * 96 - N, pad128 = ceil_div(N, 128) * 128 - N;
    const int64_t pad192 = ceil_div(N, 192) * 192 - N;
    t.bn = (pad96 < pad128) ? 96 : 128;
    if (!trans_a && K >= 2048 && pad192 <= pad96 && pad192 <= pad128 && ceil_div(M, 128) * ceil_div(N, 192) >= 512)
      t.bn = 192;
  }
  return t;
}

struct SplitChoice {
  int splits;
  int64_t k_per_split;
};

// Split-K factor.
inline SplitChoice choose_split(const rsvd_ctx *ctx, const TileChoice &t, int64_t M, int64_t N, int64_t K,
                                int force, bool upper = false, int batch = 1) {
  int64_t tiles = ceil_div(M, t.bm) * ceil_div(N, t.bn);
  if (upper) {                     // only tiles that reach the diagonal or lie above it do work
    tiles = 0;
    for (int64_t tm = 0; tm < ceil_div(M, t.bm); ++tm)
      for (int64_t tn = 0; tn < ceil_div(N, t.bn); ++tn)
        if ((tn + 1) * t.bn > tm * t.bm) ++tiles;
  }
  const int64_t ktiles = ceil_div(K, 32);
  int64_t s = 1;
  if (force > 0) {
    s = force;
  } else {
    // Aim at four workgroups per CU (measured better than two from l = 16, where the kernels are HBM
    // bound and need the loads in flight, to l = 576), rounded to the nearest factor so that a grid
    // that nearly fills the chip is left alone.  Every split pays a prologue and a tile-sized
    // partial store: at least 4 k-tiles per split for the 64-row tiles (2 for a small Gram matrix, whose few
    // workgroups are bound by the chain of dependent loads, one per k-tile), 8 for the larger ones.
    const int64_t want = 4 * (int64_t)ctx->cu_count;
    tiles *= batch;                  // a batch fills the chip with fewer splits per problem
    if (tiles < want) s = (want + tiles / 2) / tiles;
    const int64_t min_k = (t.bm * t.bn > 64 * 128) ? 8 : (M == N && M <= 128 ? 2 : 4);
    const int64_t max_by_k = ktiles / min_k > 0 ? ktiles / min_k : 1;
    if (s > max_by_k) s = max_by_k;
    if (s > 256) s = 256;
    if (s < 1) s = 1;
  }
  if (s > ktiles) s = ktiles > 0 ? ktiles : 1;
  SplitChoice c;
  c.k_per_split = ceil_div(ktiles, s) * 32;
  c.splits = (int)ceil_div(K, c.k_per_split);
  if (c.splits < 1) c.splits = 1;
  return c;
}

template <typename TAcc, typename TOut>
inline void launch_plain_reduce(hipStream_t s, const GemmParams &P, unsigned blocks, unsigned batch) {
  if constexpr (sizeof(TAcc) == sizeof(TOut)) {
    hipLaunchKernelGGL((splitk_reduce_plain_kernel<TAcc, TOut>), dim3(blocks, batch), dim3(256), 0, s, P);
  }
}

template <typename TIn, typename TAcc, typename TOut>
struct GemmDispatch {
  template <bool TA, int BM, int BN, int WGM, int WGN, int BK = 32>
  static hipError_t run(hipStream_t s, const GemmParams &P, bool vec, int batch) {
    GemmParams Q = P;
    Q.tiles_n = (int)ceil_div(P.N, BN);
    Q.tiles_m = (int)ceil_div(P.M, BM);
    dim3 grid((unsigned)((int64_t)Q.tiles_n * Q.tiles_m * P.splits), (unsigned)batch);
    constexpr int V = 16 / sizeof(TIn);
    const bool general = P.splits == 1 && (P.dead != nullptr || P.trans_c != 0);
    const bool scaled = P.splits == 1 && !general && (P.alpha != 1.0 || P.beta != 0.0);
    if (P.a_shift != nullptr) {
      if (vec) hipLaunchKernelGGL((gemm_kernel<TIn, TAcc, TOut, TA, BM, BN, WGM, WGN, V, 3, BK>), grid, dim3(256), 0, s, Q);
      else hipLaunchKernelGGL((gemm_kernel<TIn, TAcc, TOut, TA, BM, BN, WGM, WGN, 1, 3, BK>), grid, dim3(256), 0, s, Q);
    } else if (general) {
      if (vec) hipLaunchKernelGGL((gemm_kernel<TIn, TAcc, TOut, TA, BM, BN, WGM, WGN, V, 1, BK>), grid, dim3(256), 0, s, Q);
      else hipLaunchKernelGGL((gemm_kernel<TIn, TAcc, TOut, TA, BM, BN, WGM, WGN, 1, 1, BK>), grid, dim3(256), 0, s, Q);
    } else if (scaled) {
      if (vec) hipLaunchKernelGGL((gemm_kernel<TIn, TAcc, TOut, TA, BM, BN, WGM, WGN, V, 2, BK>), grid, dim3(256), 0, s, Q);
      else hipLaunchKernelGGL((gemm_kernel<TIn, TAcc, TOut, TA, BM, BN, WGM, WGN, 1, 2, BK>), grid, dim3(256), 0, s, Q);
    } else {
      if (vec) hipLaunchKernelGGL((gemm_kernel<TIn, TAcc, TOut, TA, BM, BN, WGM, WGN, V, 0, BK>), grid, dim3(256), 0, s, Q);
      else hipLaunchKernelGGL((gemm_kernel<TIn, TAcc, TOut, TA, BM, BN, WGM, WGN, 1, 0, BK>), grid, dim3(256), 0, s, Q);
    }
    return hipGetLastError();
  }

  template <bool TA>
  static hipError_t by_tile(hipStream_t s, const GemmParams &P, const TileChoice &t, bool vec, int batch) {
    if (t.bm == 64) {
      switch (t.bn) {
        // (64-deep k-tiles for these HBM-bound shapes measured no better than 32)
        case 16:  return run<TA, 64, 16, 4, 1>(s, P, vec, batch);
        case 32:  return run<TA, 64, 32, 4, 1>(s, P, vec, batch);
        case 48:  return run<TA, 64, 48, 4, 1>(s, P, vec, batch);
        case 64:  return run<TA, 64, 64, 4, 1>(s, P, vec, batch);
        case 80:  return run<TA, 64, 80, 4, 1>(s, P, vec, batch);
        case 96:  return run<TA, 64, 96, 4, 1>(s, P, vec, batch);
        case 112: return run<TA, 64, 112, 4, 1>(s, P, vec, batch);
        case 128: return run<TA, 64, 128, 4, 1>(s, P, vec, batch);
      }
    } else {
      if (t.bn == 96)  return run<TA, 128, 96, 2, 2>(s, P, vec, batch);
      if (t.bn == 128) return run<TA, 128, 128, 2, 2>(s, P, vec, batch);
      if (t.bn == 192 && sizeof(TAcc) == 4) return run<TA, 128, 192, 2, 2>(s, P, vec, batch);
    }
    return hipErrorInvalidValue;
  }

  static size_t partial_bytes(const rsvd_ctx *ctx, int64_t M, int64_t N, int64_t K, bool trans_a) {
    const TileChoice t = choose_tile(M, N, K, sizeof(TAcc), trans_a);
    SplitChoice c = choose_split(ctx, t, M, N, K, 0);
    if (M == N) {                  // a symmetric (upper-only) product of this shape may split further
      const SplitChoice cu = choose_split(ctx, choose_tile(M, N, K, sizeof(TAcc), trans_a, true), M, N, K, 0, true);
      if (cu.splits > c.splits) c = cu;
    }
    return c.splits > 1 ? (size_t)c.splits * (size_t)M * (size_t)N * sizeof(TAcc) : 0;
  }

  static hipError_t launch(rsvd_ctx *ctx, hipStream_t s, const GemmDesc &d) {
    if (d.M <= 0 || d.N <= 0) return hipSuccess;
    const TileChoice t = choose_tile(d.M, d.N, d.K, sizeof(TAcc), d.trans_a != 0, d.upper_only != 0);
    if (d.batch < 1 || d.batch > 65535) return hipErrorInvalidValue;
    SplitChoice c = choose_split(ctx, t, d.M, d.N, d.K, d.force_splits, d.upper_only != 0, d.batch);
    if (c.splits > 1) {
      const size_t need = (size_t)c.splits * (size_t)d.M * (size_t)d.N * sizeof(TAcc);
      if (d.partial == nullptr || d.partial_bytes < need) return hipErrorInvalidValue;
    }
    if (d.trans_c && d.beta != 0.0) return hipErrorInvalidValue;
    // the centred product has the lean epilogue only
    if (d.a_shift != nullptr && (d.dead != nullptr || d.trans_c || d.alpha != 1.0 || d.beta != 0.0 || d.batch != 1))
      return hipErrorInvalidValue;
    GemmParams P;
    P.M = d.M; P.N = d.N; P.K = d.K;
    P.A = d.A; P.lda = d.lda; P.B = d.B; P.ldb = d.ldb; P.C = d.C; P.ldc = d.ldc;
    P.partial = d.partial; P.k_per_split = c.k_per_split; P.splits = c.splits;
    P.trans_c = d.trans_c; P.alpha = d.alpha; P.beta = d.beta;
    P.upper_bm = d.upper_only ? t.bm : 0; P.upper_bn = d.upper_only ? t.bn : 0;
    P.b_upper = d.b_upper;
    P.a_shift = d.a_shift;
    P.dead = d.dead; P.seed = d.seed; P.refill_stream = d.refill_stream;
    P.refill_scale = d.refill_scale; P.refill_ld = d.refill_ld;
    P.stride_a = d.stride_a; P.stride_b = d.stride_b; P.stride_c = d.stride_c; P.stride_partial = d.stride_partial;
    P.stride_dead = d.stride_dead; P.seed_step = d.seed_step;
    P.skip_flag = d.skip_flag; P.alt_flag = d.alt_flag; P.B_alt = d.B_alt; P.stride_flag = d.stride_flag; P.skip_now = 0;
    P.reduce_groups = 1;
    // 16-byte vector loads need aligned bases, leading dimensions and extents.
    constexpr int V = 16 / sizeof(TIn);
    const int64_t a_contig = d.trans_a ? d.M : d.K;
    const bool vec = ((uintptr_t)d.A % 16 == 0) && ((uintptr_t)d.B % 16 == 0) && d.lda % V == 0 &&
                     d.ldb % V == 0 && a_contig % V == 0 && d.N % V == 0 &&
                     (d.batch == 1 || (d.stride_a % 16 == 0 && d.stride_b % 16 == 0)) &&
                     (d.B_alt == nullptr || (uintptr_t)d.B_alt % 16 == 0);
    hipError_t e;
    {
      ProfScope ps(ctx, s, d.prof_kind);
      e = d.trans_a ? by_tile<true>(s, P, t, vec, d.batch) : by_tile<false>(s, P, t, vec, d.batch);
    }
    if (e != hipSuccess) return e;
    if (d.splits_out != nullptr) *d.splits_out = c.splits;
    if (c.splits > 1 && !(d.skip_reduce && c.splits <= d.skip_reduce_max)) {
      ProfScope ps(ctx, s, d.prof_kind + 1);
      constexpr int V16 = 16 / sizeof(TAcc);
      const bool plain = sizeof(TAcc) == sizeof(TOut) && d.alpha == 1.0 && d.beta == 0.0 && d.dead == nullptr &&
                         !d.trans_c && !d.upper_only && d.N % V16 == 0 && d.ldc % V16 == 0 &&
                         (uintptr_t)d.C % 16 == 0 && (uintptr_t)d.partial % 16 == 0 &&
                         (d.batch == 1 || (d.stride_c % 16 == 0 && d.stride_partial % 16 == 0)) &&
                         d.M * d.N >= 262144;       // (smaller outputs do better with one element per thread)
      if (plain) {
        int64_t blocks = ceil_div(d.M * d.N / V16, 256);
        if (blocks > 8192) blocks = 8192;
        launch_plain_reduce<TAcc, TOut>(s, P, (unsigned)blocks, (unsigned)d.batch);
        return hipGetLastError();
      }
      // threads per element: enough of them to put ~64k loads in flight, at least eight partials each
      int sg = 1;
      while (sg < 8 && d.M * d.N * d.batch * sg < 65536 && c.splits >= 16 * sg) sg *= 2;
      P.reduce_groups = sg;
      int64_t blocks = ceil_div(d.M * d.N, 256 / sg);
      if (blocks > 8192) blocks = 8192;
      hipLaunchKernelGGL((splitk_reduce_kernel<TIn, TAcc, TOut>), dim3((unsigned)blocks, (unsigned)d.batch), dim3(256),
                         0, s, P);
      e = hipGetLastError();
    }
    return e;
  }
};

}  // namespace rsvd
