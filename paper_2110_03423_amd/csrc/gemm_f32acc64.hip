// GEMM instantiation: inputs float, MFMA accumulator double, output double.
#include "gemm_impl.hpp"

namespace rsvd {
size_t gemm_partial_bytes_f32acc64(const rsvd_ctx *ctx, int64_t M, int64_t N, int64_t K, int trans_a) {
  return GemmDispatch<float, double, double>::partial_bytes(ctx, M, N, K, trans_a != 0);
}
hipError_t gemm_launch_f32acc64(rsvd_ctx *ctx, hipStream_t s, const GemmDesc &d) {
  return GemmDispatch<float, double, double>::launch(ctx, s, d);
}
}  // namespace rsvd
