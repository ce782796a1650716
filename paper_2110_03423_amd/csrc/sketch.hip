// Step 1 of Algorithm 1: the Gaussian sketching matrix, generated on the device.
#include "common.hpp"
#include "philox_dev.hpp"

namespace rsvd {

// One thread per Philox group; the group's 4 (fp32) or 2 (fp64) normals go to
// consecutive row-major elements of the rows x cols matrix.  Problem blockIdx.y of a batch
// uses seed + blockIdx.y and writes stride_out bytes further on.
template <typename T, bool F32>
__global__ __launch_bounds__(256) void sketch_kernel(uint64_t seed, uint32_t stream, int64_t cols,
                                                     int64_t total, T *__restrict__ out, int64_t ld,
                                                     int64_t stride_out) {
  constexpr int PER = F32 ? 4 : 2;
  seed += (uint64_t)blockIdx.y;
  out = reinterpret_cast<T *>(reinterpret_cast<char *>(out) + (int64_t)blockIdx.y * stride_out);
  const int64_t n_groups = (total + PER - 1) / PER;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < n_groups;
       g += (int64_t)gridDim.x * blockDim.x) {
    double z[4];
    philox_normals<F32>((uint64_t)g, stream, seed, z);
    const int64_t e0 = g * PER;
    int64_t i = e0 / cols;
    int64_t j = e0 - i * cols;
    if (ld == cols && e0 + PER <= total && ((reinterpret_cast<uintptr_t>(out) & 15) == 0)) {
      // dense output: one 16-byte store per group
      if (F32) {
        float4 v = make_float4((float)z[0], (float)z[1], (float)z[2], (float)z[3]);
        *reinterpret_cast<float4 *>(out + e0) = v;
      } else {
        double2 v = make_double2(z[0], z[1]);
        *reinterpret_cast<double2 *>(out + e0) = v;
      }
      continue;
    }
#pragma unroll
    for (int t = 0; t < PER; ++t) {
      if (e0 + t < total) out[i * ld + j] = (T)z[t];
      if (++j == cols) { j = 0; ++i; }
    }
  }
}

__global__ __launch_bounds__(256) void philox_raw_kernel(uint64_t seed, uint32_t stream, uint64_t first,
                                                         int64_t n_groups, uint32_t *__restrict__ out) {
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < n_groups;
       g += (int64_t)gridDim.x * blockDim.x) {
    const Philox4 p = philox4x32_10(first + (uint64_t)g, stream, seed);
#pragma unroll
    for (int t = 0; t < 4; ++t) out[g * 4 + t] = p.x[t];
  }
}

static int grid_for(int64_t items) {
  int64_t blocks = ceil_div(items, 256);
  if (blocks < 1) blocks = 1;
  if (blocks > 256 * 32) blocks = 256 * 32;
  return (int)blocks;
}

hipError_t sketch_launch(hipStream_t s, rsvd_dtype dtype, uint64_t seed, uint32_t stream_id,
                         int64_t rows, int64_t cols, void *out, int64_t ld, int batch, int64_t stride_out) {
  const int64_t total = rows * cols;
  if (total == 0) return hipSuccess;
  if (batch < 1 || batch > 65535) return hipErrorInvalidValue;
  if (dtype == RSVD_F32) {
    hipLaunchKernelGGL((sketch_kernel<float, true>), dim3(grid_for((total + 3) / 4), batch), dim3(256), 0, s,
                       seed, stream_id, cols, total, (float *)out, ld, stride_out);
  } else {
    hipLaunchKernelGGL((sketch_kernel<double, false>), dim3(grid_for((total + 1) / 2), batch), dim3(256), 0, s,
                       seed, stream_id, cols, total, (double *)out, ld, stride_out);
  }
  return hipGetLastError();
}

hipError_t philox_raw_launch(hipStream_t s, uint64_t seed, uint32_t stream_id, uint64_t first_group,
                             int64_t n_groups, uint32_t *out) {
  if (n_groups == 0) return hipSuccess;
  hipLaunchKernelGGL(philox_raw_kernel, dim3(grid_for(n_groups)), dim3(256), 0, s, seed, stream_id,
                     first_group, n_groups, out);
  return hipGetLastError();
}

}  // namespace rsvd
