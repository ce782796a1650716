// 16x16x4 matrix-core instructions of gfx950 in fp32 and fp64, with their operand
// and accumulator layouts.
#pragma once

#include <hip/hip_runtime.h>

namespace rsvd {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));

// 16x16x4 MFMA: lane L supplies A[L % 16][L / 16] and B[L / 16][L % 16];
// the 4 accumulator registers of lane L hold column L % 16 and the rows given by row().
template <typename TAcc> struct Mfma;
template <> struct Mfma<float> {
  typedef f32x4 vec;
  static __device__ __forceinline__ vec run(float a, float b, vec c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ int row(int lane, int v) { return 4 * (lane >> 4) + v; }
};
template <> struct Mfma<double> {
  typedef f64x4 vec;
  static __device__ __forceinline__ vec run(double a, double b, vec c) {
    return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ int row(int lane, int v) { return 4 * v + (lane >> 4); }
};

}  // namespace rsvd
