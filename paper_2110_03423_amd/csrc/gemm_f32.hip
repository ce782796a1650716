// GEMM instantiation: inputs float, MFMA accumulator float, output float.
#include "gemm_impl.hpp"

namespace rsvd {
size_t gemm_partial_bytes_f32(const rsvd_ctx *ctx, int64_t M, int64_t N, int64_t K, int trans_a) {
  return GemmDispatch<float, float, float>::partial_bytes(ctx, M, N, K, trans_a != 0);
}
hipError_t gemm_launch_f32(rsvd_ctx *ctx, hipStream_t s, const GemmDesc &d) {
  return GemmDispatch<float, float, float>::launch(ctx, s, d);
}
}  // namespace rsvd
