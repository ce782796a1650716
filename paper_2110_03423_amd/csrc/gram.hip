// Step 3 of Algorithm 1, the Gram matrix of CholeskyQR for panels of up to 128 columns: G = Y^T Y in fp64,
// Y rows x l in fp32 or fp64.
//
// As a general product (A = B = Y^T... the same memory read as two operands, 64 x 64 output tiles, the three tiles
// on or above the diagonal, the rows split over ~1000 workgroups that each leave a tile-sized fp64 partial sum) the
// 100000 x 120 panel took 63 + 8 us: every row of Y is fetched six times through L2 and the partial sums weigh as
// much as the panel.  Here a workgroup owns a range of rows and ALL l columns: a k-tile of 32 rows of Y goes to LDS
// once and feeds both operands of the matrix instruction; the 16 x 16 blocks on or above the diagonal
// (NBLK (NBLK + 1) / 2 of them, 36 at l = 128 where the three tiles make 48) are dealt out to the four wavefronts,
// whose fp64 accumulators stay in registers over the whole range of rows; one workgroup per CU, the next k-tile in
// flight while the matrix cores work (an fp64 matrix instruction takes 64 cycles, nine of them per lane and k-step:
// one wavefront per SIMD keeps the pipe busy).  The G workgroups leave G partial matrices, which the split-K
// reduction adds in a fixed order (or the Cholesky kernel itself, for up to four).
#include <utility>

#include "gemm_impl.hpp"

namespace rsvd {

struct SyrkParams {
  int64_t rows; int l;
  const void *Y; int64_t ldy;
  double *out;                    // [G][l][l] partial sums (G > 1), or the l x l result itself (G == 1)
  int64_t rows_per_wg;
  int64_t stride_y, stride_out;   // batched launch (blockIdx.y), bytes
  const int *skip_flag; int64_t stride_flag;
};

// Upper block triangle in row-major order: block idx -> (bi, bj), bi <= bj < NBLK.
template <int NBLK> __host__ __device__ constexpr int syrk_bi(int idx) {
  int bi = 0, left = idx;
  while (left >= NBLK - bi) { left -= NBLK - bi; ++bi; }
  return bi;
}
template <int NBLK> __host__ __device__ constexpr int syrk_bj(int idx) {
  int bi = 0, left = idx;
  while (left >= NBLK - bi) { left -= NBLK - bi; ++bi; }
  return bi + left;
}

template <int NBLK, int IDX> constexpr int kSyrkBi = syrk_bi<NBLK>(IDX);
template <int NBLK, int IDX> constexpr int kSyrkBj = syrk_bj<NBLK>(IDX);

// acc[b] += x[bi]^T x[bj] for the blocks W, W + 4, ... (indices fixed at compile time: x and acc stay in registers)
template <int NBLK, int W, int N, int... Bs>
__device__ __forceinline__ void syrk_step(const double (&x)[NBLK], f64x4 (&acc)[N], std::integer_sequence<int, Bs...>) {
  ((acc[Bs] = Mfma<double>::run(x[kSyrkBi<NBLK, W + 4 * Bs>], x[kSyrkBj<NBLK, W + 4 * Bs>], acc[Bs])), ...);
}
template <int NBLK, int W, int N, int... Bs>
__device__ __forceinline__ void syrk_store(const f64x4 (&acc)[N], double *out, int l, int lane,
                                           std::integer_sequence<int, Bs...>) {
  const int r16 = lane & 15;
  auto one = [&](int bi, int bj, const f64x4 &a) {
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = 16 * bi + Mfma<double>::row(lane, v), col = 16 * bj + r16;
      if (row < l && col < l) out[(int64_t)row * l + col] = a[v];
    }
  };
  (one(kSyrkBi<NBLK, W + 4 * Bs>, kSyrkBj<NBLK, W + 4 * Bs>, acc[Bs]), ...);
}

template <typename TIn, int NBLK> struct SyrkCfg {
  static constexpr int BK = 32, LP = 16 * NBLK, SY = LP + pad_kmajor(LP);
  static constexpr int NB2 = NBLK * (NBLK + 1) / 2, MAXB = (NB2 + 3) / 4;
  static constexpr size_t lds_bytes = (size_t)2 * BK * SY * sizeof(TIn);
};

// The work of wavefront W: blocks W, W + 4, ... of the upper triangle.
template <typename TIn, int NBLK, int VEC, int W>
__device__ __forceinline__ void syrk_wave(const SyrkParams &P, TIn *Ys, int64_t r0, int64_t r1, double *out) {
  typedef SyrkCfg<TIn, NBLK> C;
  constexpr int BK = C::BK, LP = C::LP, SY = C::SY, NB2 = C::NB2;
  constexpr int NMINE = (NB2 - W + 3) / 4;
  const int tid = threadIdx.x, lane = tid & 63;
  const int r16 = lane & 15, kq = lane >> 4;
  const TIn *Y = (const TIn *)P.Y;
  f64x4 acc[NMINE > 0 ? NMINE : 1];
#pragma unroll
  for (int b = 0; b < NMINE; ++b) acc[b] = f64x4{0.0, 0.0, 0.0, 0.0};
  TileStage<TIn, BK, LP, VEC> st;
  st.load(Y + r0 * P.ldy, P.ldy, r1 - r0, P.l, tid);
  st.store(Ys, SY, tid);
  __syncthreads();
  int buf = 0;
  for (int64_t k0 = r0; k0 < r1; k0 += BK, buf ^= 1) {
    const bool more = k0 + BK < r1;
    if (more) st.load(Y + (k0 + BK) * P.ldy, P.ldy, r1 - (k0 + BK), P.l, tid);
    const TIn *cur = Ys + buf * BK * SY + kq * SY + r16;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 4) {
      double x[NBLK];
#pragma unroll
      for (int c = 0; c < NBLK; ++c) x[c] = (double)cur[kk * SY + 16 * c];
      syrk_step<NBLK, W>(x, acc, std::make_integer_sequence<int, NMINE>());
    }
    if (more) st.store(Ys + (buf ^ 1) * BK * SY, SY, tid);
    __syncthreads();
  }
  syrk_store<NBLK, W>(acc, out, P.l, lane, std::make_integer_sequence<int, NMINE>());
}

template <typename TIn, int NBLK, int VEC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gram_syrk_kernel(const SyrkParams P0) {
  SyrkParams P = P0;
  {
    const int64_t b = (int64_t)blockIdx.y;
    if (P.skip_flag != nullptr && *(const int *)((const char *)P.skip_flag + b * P.stride_flag) != 0) return;
    P.Y = (const char *)P.Y + b * P.stride_y;
    P.out = (double *)((char *)P.out + b * P.stride_out);
  }
  extern __shared__ __attribute__((aligned(16))) double syrk_lds[];
  TIn *Ys = reinterpret_cast<TIn *>(syrk_lds);
  const int64_t r0 = (int64_t)blockIdx.x * P.rows_per_wg;
  const int64_t r1 = (r0 + P.rows_per_wg < P.rows) ? r0 + P.rows_per_wg : P.rows;
  double *out = P.out + (int64_t)blockIdx.x * P.l * P.l;
  switch (threadIdx.x >> 6) {
    case 0: syrk_wave<TIn, NBLK, VEC, 0>(P, Ys, r0, r1, out); break;
    case 1: syrk_wave<TIn, NBLK, VEC, 1>(P, Ys, r0, r1, out); break;
    case 2: syrk_wave<TIn, NBLK, VEC, 2>(P, Ys, r0, r1, out); break;
    default: syrk_wave<TIn, NBLK, VEC, 3>(P, Ys, r0, r1, out); break;
  }
}

// Rows per workgroup and number of workgroups: one workgroup per CU when the panel is long enough for that; a short
// panel is cut so that a workgroup works for ~3 us (a k-tile of 32 rows takes 2.2 us of matrix instructions at
// l = 128, where a wavefront has nine blocks, in proportion less below, and never less than its loads take), since
// every workgroup pays for the l x l partial sum it leaves.
static void syrk_split(const rsvd_ctx *ctx, int64_t rows, int64_t l, int64_t &rows_per_wg, int &wgs) {
  const int64_t nblk = ceil_div(l, 16), nb2 = nblk * (nblk + 1) / 2;
  double per_ktile = 2.2 * (double)nb2 / 36.0;          // us; never less than the ~0.6 us a k-tile's loads take
  if (per_ktile < 0.6) per_ktile = 0.6;
  int64_t ktiles = (int64_t)(3.0 / per_ktile);
  if (ktiles < 1) ktiles = 1;
  rows_per_wg = ceil_div(ceil_div(rows, (int64_t)ctx->cu_count), 32) * 32;
  if (rows_per_wg < 32 * ktiles) rows_per_wg = 32 * ktiles;
  wgs = (int)ceil_div(rows, rows_per_wg);
  if (wgs < 1) wgs = 1;
}

int gram_syrk_max_order() { return 128; }

size_t gram_syrk_partial_bytes(const rsvd_ctx *ctx, int64_t rows, int64_t l) {
  if (l > gram_syrk_max_order()) return 0;
  int64_t rpw; int wgs;
  syrk_split(ctx, rows, l, rpw, wgs);
  return wgs > 1 ? (size_t)wgs * (size_t)l * (size_t)l * sizeof(double) : 0;
}

template <typename TIn, int NBLK>
static void syrk_raise_lds(hipError_t &e) {
  constexpr int V = 16 / sizeof(TIn);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gram_syrk_kernel<TIn, NBLK, V>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)SyrkCfg<TIn, NBLK>::lds_bytes);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&gram_syrk_kernel<TIn, NBLK, 1>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)SyrkCfg<TIn, NBLK>::lds_bytes);
}
template <typename TIn>
static void syrk_raise_all(hipError_t &e) {
  syrk_raise_lds<TIn, 1>(e); syrk_raise_lds<TIn, 2>(e); syrk_raise_lds<TIn, 3>(e); syrk_raise_lds<TIn, 4>(e);
  syrk_raise_lds<TIn, 5>(e); syrk_raise_lds<TIn, 6>(e); syrk_raise_lds<TIn, 7>(e); syrk_raise_lds<TIn, 8>(e);
}
hipError_t gram_init_device(rsvd_ctx *ctx) {
  (void)ctx;
  hipError_t e = hipSuccess;
  syrk_raise_all<float>(e);
  syrk_raise_all<double>(e);
  return e;
}

template <typename TIn, int NBLK>
static hipError_t syrk_run(hipStream_t s, const SyrkParams &P, int wgs, int batch, bool vec) {
  constexpr int V = 16 / sizeof(TIn);
  const size_t lds = SyrkCfg<TIn, NBLK>::lds_bytes;
  if (vec) hipLaunchKernelGGL((gram_syrk_kernel<TIn, NBLK, V>), dim3(wgs, batch), dim3(256), lds, s, P);
  else hipLaunchKernelGGL((gram_syrk_kernel<TIn, NBLK, 1>), dim3(wgs, batch), dim3(256), lds, s, P);
  return hipGetLastError();
}
template <typename TIn>
static hipError_t syrk_by_order(hipStream_t s, const SyrkParams &P, int wgs, int batch, bool vec) {
  switch ((P.l + 15) / 16) {
    case 1: return syrk_run<TIn, 1>(s, P, wgs, batch, vec);
    case 2: return syrk_run<TIn, 2>(s, P, wgs, batch, vec);
    case 3: return syrk_run<TIn, 3>(s, P, wgs, batch, vec);
    case 4: return syrk_run<TIn, 4>(s, P, wgs, batch, vec);
    case 5: return syrk_run<TIn, 5>(s, P, wgs, batch, vec);
    case 6: return syrk_run<TIn, 6>(s, P, wgs, batch, vec);
    case 7: return syrk_run<TIn, 7>(s, P, wgs, batch, vec);
    case 8: return syrk_run<TIn, 8>(s, P, wgs, batch, vec);
  }
  return hipErrorInvalidValue;
}

// G = Y^T Y (upper 16 x 16 blocks; what lies in the blocks below the diagonal is left as it was).  *parts_out
// receives the number of partial matrices left in `partial` for the consumer to add (1: Gout holds the result):
// up to max_parts of them are left, more are added here into Gout.
hipError_t gram_syrk_launch(rsvd_ctx *ctx, hipStream_t s, rsvd_dtype dtype, int64_t rows, int64_t l, const void *Y,
                            int64_t ldy, double *Gout, void *partial, size_t partial_bytes, int max_parts,
                            int *parts_out, int batch, int64_t stride, const int *skip_flag) {
  if (l < 1 || l > gram_syrk_max_order() || rows < 1 || batch < 1 || batch > 65535) return hipErrorInvalidValue;
  int64_t rpw; int wgs;
  syrk_split(ctx, rows, l, rpw, wgs);
  if (wgs > 1 && (partial == nullptr || partial_bytes < (size_t)wgs * l * l * sizeof(double))) return hipErrorInvalidValue;
  SyrkParams P;
  P.rows = rows; P.l = (int)l; P.Y = Y; P.ldy = ldy;
  P.out = wgs > 1 ? (double *)partial : Gout;
  P.rows_per_wg = rpw;
  P.stride_y = stride; P.stride_out = stride;
  P.skip_flag = skip_flag; P.stride_flag = stride;
  const int64_t V = 16 / (int64_t)dtype_size(dtype);
  const bool vec = ((uintptr_t)Y % 16 == 0) && ldy % V == 0 && l % V == 0 && (batch == 1 || stride % 16 == 0);
  hipError_t e;
  {
    ProfScope ps(ctx, s, PK_GRAM);
    e = dtype == RSVD_F32 ? syrk_by_order<float>(s, P, wgs, batch, vec) : syrk_by_order<double>(s, P, wgs, batch, vec);
  }
  if (e != hipSuccess) return e;
  if (parts_out != nullptr) *parts_out = wgs;
  if (wgs > 1 && wgs > max_parts) {
    // the split-K reduction of the product kernels, told which 16 x 16 blocks exist
    GemmParams R;
    R.M = l; R.N = l; R.K = rows;
    R.A = nullptr; R.lda = 0; R.B = nullptr; R.ldb = 0; R.C = Gout; R.ldc = l;
    R.partial = partial; R.k_per_split = 0; R.splits = wgs;
    R.tiles_n = R.tiles_m = 0; R.upper_bm = 16; R.upper_bn = 16; R.b_upper = 0;
    R.trans_c = 0; R.alpha = 1.0; R.beta = 0.0; R.a_shift = nullptr; R.dead = nullptr;
    R.seed = 0; R.refill_stream = 0; R.refill_scale = 1.0; R.refill_ld = 0;
    R.stride_a = R.stride_b = 0; R.stride_c = stride; R.stride_partial = stride; R.stride_dead = 0; R.seed_step = 0;
    R.skip_flag = skip_flag; R.alt_flag = nullptr; R.B_alt = nullptr; R.stride_flag = stride; R.skip_now = 0;
    int sg = 1;
    while (sg < 8 && l * l * batch * sg < 65536 && wgs >= 16 * sg) sg *= 2;
    R.reduce_groups = sg;
    int64_t blocks = ceil_div(l * l, (int64_t)(256 / sg));
    if (blocks > 8192) blocks = 8192;
    ProfScope ps(ctx, s, PK_GRAM_REDUCE);
    hipLaunchKernelGGL((splitk_reduce_kernel<double, double, double>), dim3((unsigned)blocks, (unsigned)batch), dim3(256),
                       0, s, R);
    e = hipGetLastError();
    if (parts_out != nullptr) *parts_out = 1;
  }
  return e;
}

}  // namespace rsvd
