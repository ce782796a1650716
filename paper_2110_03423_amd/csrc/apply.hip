// Step 3 of Algorithm 1, the triangular apply of CholeskyQR for panels of up to 128 columns:
// Q = Y R^-1 with Y rows x l and R^-1 l x l upper triangular.
//
// The general product kernel treats this as any other GEMM: one workgroup per 64-row tile, R^-1 pulled from L2 again
// by every workgroup, k-tile by k-tile, with as many exposed load latencies as there are k-tiles (four at l = 120)
// and no use of the zeros below the diagonal; on the 100000 x 120 panel it ran at a quarter of the memory rate.
// Here every wavefront keeps its share of R^-1 in registers, in the B-operand layout of the matrix instruction
// (the upper triangle only: 144 values per lane at l = 128), so that only the rows of Y pass through LDS; a
// workgroup walks over row tiles (workgroup g takes tiles g, g + G, ...), has the next tile's rows in flight while
// the matrix cores work on the current one, and issues only the matrix instructions whose k range reaches the column
// block (4 (j + 1) of them for block j instead of 4 NBLK).  One workgroup per CU, one wavefront per SIMD (the
// registers: 144 for R^-1, 32 each for the accumulators, the A operands of a tile and the rows in flight); the tile
// buffer in LDS is double, so that a tile costs one barrier.  (R^-1 in LDS instead: one LDS read per matrix
// instruction, no faster than the general kernel; two workgroups per CU: the 256 registers left per wavefront
// spill.)  The result may overwrite Y: a tile's rows are complete in LDS before the first of them is stored.
// Columns flagged as dependent are replaced by fresh Gaussian directions, as in the general kernel's epilogue.
#include "gemm_impl.hpp"

namespace rsvd {

struct ApplyParams {
  int64_t rows; int l;
  const void *Y; int64_t ldy;
  const void *Rinv;                      // l x l, ld l
  void *Q; int64_t ldq;
  const int *dead;
  uint64_t seed; uint32_t refill_stream; double refill_scale; int64_t refill_ld;
  int64_t stride_y, stride_r, stride_q, stride_dead; uint64_t seed_step;      // batched launch (blockIdx.y), bytes
  const int *skip_flag; int64_t stride_flag;
  int tiles;
};

template <typename T, int NBLK> struct ApplyLds {
  static constexpr int LP = 16 * NBLK;
  static constexpr int SA = LP + (sizeof(T) == 4 ? 4 : 2);
  static constexpr size_t bytes = (size_t)2 * 64 * SA * sizeof(T);
};

template <typename T, int NBLK, int VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void apply_tri_kernel(const ApplyParams P0) {
  ApplyParams P = P0;
  {
    const int64_t b = (int64_t)blockIdx.y;
    if (P.skip_flag != nullptr && *(const int *)((const char *)P.skip_flag + b * P.stride_flag) != 0) return;
    P.Y = (const char *)P.Y + b * P.stride_y;
    P.Rinv = (const char *)P.Rinv + b * P.stride_r;
    P.Q = (char *)P.Q + b * P.stride_q;
    if (P.dead != nullptr) P.dead = (const int *)((const char *)P.dead + b * P.stride_dead);
    P.seed += (uint64_t)b * P.seed_step;
  }
  typedef ApplyLds<T, NBLK> L;
  constexpr int LP = L::LP, SA = L::SA;
  extern __shared__ __attribute__((aligned(16))) double apply_lds[];
  T *As = reinterpret_cast<T *>(apply_lds);          // two tiles of Y, [64][SA] row-major each

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kq = lane >> 4;
  const int l = P.l;
  const T *Y = (const T *)P.Y;
  T *Q = (T *)P.Q;

  TileStage<T, 64, LP, VEC> st;
  int tile = (int)blockIdx.x;
  const int G = (int)gridDim.x;
  st.load(Y + (int64_t)tile * 64 * P.ldy, P.ldy, P.rows - (int64_t)tile * 64, l, tid);       // (the grid has no more workgroups than tiles)
  // the dependent columns among this lane's NBLK columns (all flags loaded at once: behind a branch each would
  // wait for its own round trip)
  int flag[NBLK];
#pragma unroll
  for (int j = 0; j < NBLK; ++j) {
    const int col = j * 16 + r16;
    flag[j] = (P.dead != nullptr) ? P.dead[col < l ? col : l - 1] : 0;
  }
  // R^-1 as B operands, breg[s][j] = R^-1[4 s + kq][16 j + r16] for the column blocks j that k-step s reaches:
  // 64 rows of it at a time through LDS (coalesced loads, all of them in flight before the first LDS store),
  // from there into the registers
  T breg[4 * NBLK][NBLK];
  {
    const T *R = (const T *)P.Rinv;
    constexpr int CH = (LP + 63) / 64;
    T v[CH][LP / 4];
#pragma unroll
    for (int c = 0; c < CH; ++c)
#pragma unroll
      for (int u = 0; u < LP / 4; ++u) {
        const int idx = tid + 256 * u;
        const int kk = idx / LP, n = idx - kk * LP, k = 64 * c + kk;
        const bool in = k < l && n < l && k <= n;
        const T x = R[in ? (int64_t)k * l + n : 0];
        v[c][u] = in ? x : (T)0;
      }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
#pragma unroll
      for (int u = 0; u < LP / 4; ++u) {
        const int idx = tid + 256 * u;
        const int kk = idx / LP, n = idx - kk * LP;
        As[kk * SA + n] = v[c][u];
      }
      __syncthreads();
#pragma unroll
      for (int s = 16 * c; s < 16 * c + 16 && s < 4 * NBLK; ++s)
#pragma unroll
        for (int j = s / 4; j < NBLK; ++j) breg[s][j] = As[(4 * s + kq - 64 * c) * SA + 16 * j + r16];
      __syncthreads();
    }
  }
  unsigned dead_cols = 0u;
#pragma unroll
  for (int j = 0; j < NBLK; ++j)
    if (j * 16 + r16 < l && flag[j] != 0) dead_cols |= 1u << j;
  typedef typename Mfma<T>::vec acc_t;
  st.store(As, SA, tid);
  if (tile + G < P.tiles) st.load(Y + (int64_t)(tile + G) * 64 * P.ldy, P.ldy, P.rows - (int64_t)(tile + G) * 64, l, tid);
  __syncthreads();
  for (int buf = 0; tile < P.tiles; tile += G, buf ^= 1) {
    // on entry: this tile is in As[buf], the next one (if any) in the registers of st
    const int64_t m0 = (int64_t)tile * 64;
    T *cur = As + buf * 64 * SA;
    if (tile + G < P.tiles) {
      st.store(As + (buf ^ 1) * 64 * SA, SA, tid);
      if (tile + 2 * G < P.tiles)
        st.load(Y + (int64_t)(tile + 2 * G) * 64 * P.ldy, P.ldy, P.rows - (int64_t)(tile + 2 * G) * 64, l, tid);
    }
    T a[4 * NBLK];
    const T *ap = cur + (wave * 16 + r16) * SA + kq;
#pragma unroll
    for (int s = 0; s < 4 * NBLK; ++s) a[s] = ap[4 * s];
    acc_t acc[NBLK];
#pragma unroll
    for (int j = 0; j < NBLK; ++j) acc[j] = (acc_t)(T)0;
#pragma unroll
    for (int s = 0; s < 4 * NBLK; ++s)
#pragma unroll
      for (int j = s / 4; j < NBLK; ++j) acc[j] = Mfma<T>::run(a[s], breg[s][j], acc[j]);      // k <= column only
    // The result goes back through the wavefront's own 16 rows of the tile buffer (its A operands are all in
    // registers by now) and leaves as whole rows, 16 bytes per lane: stored from the accumulator layout, 64-byte
    // pieces of four different rows per instruction, the panel was written at a third of the rate it is read at.
    T *mine = cur + (wave * 16) * SA;
#pragma unroll
    for (int j = 0; j < NBLK; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) mine[Mfma<T>::row(lane, v) * SA + j * 16 + r16] = acc[j][v];
    if (dead_cols != 0u) {
#pragma unroll 1
      for (int e = 0; e < NBLK * 4; ++e) {
        const int v = e & 3, j = e >> 2;
        if (!((dead_cols >> j) & 1u)) continue;
        const int rl = Mfma<T>::row(lane, v);
        const int64_t row = m0 + wave * 16 + rl;
        const int col = j * 16 + r16;
        mine[rl * SA + col] = (T)(P.refill_scale * philox_normal_at<sizeof(T) == 4>((uint64_t)(row * P.refill_ld + col),
                                                                                 P.refill_stream, P.seed));
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    {
      constexpr int SPR = LP / VEC;                    // slots per row
      typedef T vec_t __attribute__((ext_vector_type(VEC)));
#pragma unroll
      for (int u = 0; u < (16 * SPR + 63) / 64; ++u) {
        const int idx = lane + 64 * u;
        const int rl = idx / SPR, c = (idx - rl * SPR) * VEC;
        const int64_t row = m0 + wave * 16 + rl;
        if (idx < 16 * SPR && row < P.rows && c < l) {
          if (VEC == 1) Q[row * P.ldq + c] = mine[rl * SA + c];
          else *reinterpret_cast<vec_t *>(Q + row * P.ldq + c) = *reinterpret_cast<const vec_t *>(mine + rl * SA + c);
        }
      }
    }
    __syncthreads();          // the next tile is complete in LDS, and this one has been read by every wavefront
  }
}

template <typename T, int NBLK>
static hipError_t apply_run(const rsvd_ctx *ctx, hipStream_t s, ApplyParams P, int batch, bool vec) {
  typedef ApplyLds<T, NBLK> L;
  // one workgroup per CU: a wavefront has its SIMD, and all of its registers, to itself
  int grid = ctx->cu_count;
  if (grid > P.tiles) grid = P.tiles;
  constexpr int V = 16 / sizeof(T);
  if (vec) hipLaunchKernelGGL((apply_tri_kernel<T, NBLK, V>), dim3(grid, batch), dim3(256), L::bytes, s, P);
  else hipLaunchKernelGGL((apply_tri_kernel<T, NBLK, 1>), dim3(grid, batch), dim3(256), L::bytes, s, P);
  return hipGetLastError();
}

template <typename T, int NBLK>
static void apply_raise_lds(hipError_t &e) {
  constexpr int V = 16 / sizeof(T);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&apply_tri_kernel<T, NBLK, V>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)ApplyLds<T, NBLK>::bytes);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&apply_tri_kernel<T, NBLK, 1>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)ApplyLds<T, NBLK>::bytes);
}

// Largest l the kernel above takes (the upper triangle of R^-1 in the registers of a wavefront).
int apply_tri_max_order(rsvd_dtype dtype) { return dtype == RSVD_F32 ? 128 : 96; }

hipError_t apply_init_device(rsvd_ctx *ctx) {
  (void)ctx;
  hipError_t e = hipSuccess;
  apply_raise_lds<float, 1>(e); apply_raise_lds<float, 2>(e); apply_raise_lds<float, 3>(e); apply_raise_lds<float, 4>(e);
  apply_raise_lds<float, 5>(e); apply_raise_lds<float, 6>(e); apply_raise_lds<float, 7>(e); apply_raise_lds<float, 8>(e);
  apply_raise_lds<double, 1>(e); apply_raise_lds<double, 2>(e); apply_raise_lds<double, 3>(e);
  apply_raise_lds<double, 4>(e); apply_raise_lds<double, 5>(e); apply_raise_lds<double, 6>(e);
  return e;
}

hipError_t apply_tri_launch(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype dtype, int64_t rows, int64_t l, const void *Y,
                            int64_t ldy, const void *Rinv, void *Q, int64_t ldq, const int *dead, uint64_t seed,
                            uint32_t refill_stream, double refill_scale, int64_t refill_ld, int batch, int64_t stride,
                            const int *skip_flag) {
  if (rows <= 0 || l <= 0) return hipSuccess;
  if (l > apply_tri_max_order(dtype) || batch < 1 || batch > 65535) return hipErrorInvalidValue;
  ApplyParams P;
  P.rows = rows; P.l = (int)l; P.Y = Y; P.ldy = ldy; P.Rinv = Rinv; P.Q = Q; P.ldq = ldq; P.dead = dead;
  P.seed = seed; P.refill_stream = refill_stream; P.refill_scale = refill_scale; P.refill_ld = refill_ld;
  P.stride_y = P.stride_r = P.stride_q = P.stride_dead = stride; P.seed_step = 1;
  P.skip_flag = skip_flag; P.stride_flag = stride;
  P.tiles = (int)ceil_div(rows, 64);
  const size_t es = dtype_size(dtype);
  const int64_t V = 16 / (int64_t)es;
  const bool vec = ((uintptr_t)Y % 16 == 0) && ((uintptr_t)Q % 16 == 0) && ldy % V == 0 && ldq % V == 0 && l % V == 0 &&
                   (batch == 1 || stride % 16 == 0);
  const int nblk = (int)ceil_div(l, 16);
  ProfScope ps(ctx, s, PK_APPLY);
  if (dtype == RSVD_F32) {
    switch (nblk) {
      case 1: return apply_run<float, 1>(ctx, s, P, batch, vec);
      case 2: return apply_run<float, 2>(ctx, s, P, batch, vec);
      case 3: return apply_run<float, 3>(ctx, s, P, batch, vec);
      case 4: return apply_run<float, 4>(ctx, s, P, batch, vec);
      case 5: return apply_run<float, 5>(ctx, s, P, batch, vec);
      case 6: return apply_run<float, 6>(ctx, s, P, batch, vec);
      case 7: return apply_run<float, 7>(ctx, s, P, batch, vec);
      case 8: return apply_run<float, 8>(ctx, s, P, batch, vec);
    }
  } else {
    switch (nblk) {
      case 1: return apply_run<double, 1>(ctx, s, P, batch, vec);
      case 2: return apply_run<double, 2>(ctx, s, P, batch, vec);
      case 3: return apply_run<double, 3>(ctx, s, P, batch, vec);
      case 4: return apply_run<double, 4>(ctx, s, P, batch, vec);
      case 5: return apply_run<double, 5>(ctx, s, P, batch, vec);
      case 6: return apply_run<double, 6>(ctx, s, P, batch, vec);
    }
  }
  return hipErrorInvalidValue;
}

}  // namespace rsvd
