// Device-side Philox4x32-10 and the Gaussian transform of the sketch
// (Algorithm 1 step 1: the sketching matrix is Gaussian and drawn on the device).
//
// Stream layout (this library's own; not compatible with any vendor generator):
//   key     = (seed lo, seed hi)
//   counter = (g lo, g hi, stream, 0), g = group index
//   fp32: element e -> group e >> 2, lane e & 3; 24-bit uniforms, two Box-Muller pairs per group
//   fp64: element e -> group e >> 1, lane e & 1; 52-bit uniforms, one Box-Muller pair per group
// The Gaussian transform runs in fp64 for both output types and is rounded once.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rsvd {

struct Philox4 {
  uint32_t x[4];
};

__device__ __forceinline__ Philox4 philox4x32_10(uint64_t group, uint32_t stream, uint64_t seed) {
  uint32_t c0 = (uint32_t)group, c1 = (uint32_t)(group >> 32), c2 = stream, c3 = 0u;
  uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  Philox4 o;
  o.x[0] = c0; o.x[1] = c1; o.x[2] = c2; o.x[3] = c3;
  return o;
}

__device__ __forceinline__ double uniform24(uint32_t x) {
  return ((double)(x >> 8) + 0.5) * 0x1p-24;
}
__device__ __forceinline__ double uniform52(uint32_t hi, uint32_t lo) {
  const uint64_t v = (((uint64_t)hi << 32) | (uint64_t)lo) >> 12;
  return ((double)v + 0.5) * 0x1p-52;
}

// Box-Muller: r = sqrt(-2 ln u), angle = fl(2 pi) * v.
__device__ __forceinline__ void box_muller(double u, double v, double &z0, double &z1) {
  const double r = sqrt(-2.0 * log(u));
  const double t = 6.283185307179586 * v;
  double sn, cs;
  sincos(t, &sn, &cs);
  z0 = r * cs;
  z1 = r * sn;
}

// All normals of one group: 4 for fp32 output, 2 for fp64 output.
template <bool F32>
__device__ __forceinline__ void philox_normals(uint64_t group, uint32_t stream, uint64_t seed, double *z) {
  const Philox4 p = philox4x32_10(group, stream, seed);
  if (F32) {
    box_muller(uniform24(p.x[0]), uniform24(p.x[1]), z[0], z[1]);
    box_muller(uniform24(p.x[2]), uniform24(p.x[3]), z[2], z[3]);
  } else {
    box_muller(uniform52(p.x[0], p.x[1]), uniform52(p.x[2], p.x[3]), z[0], z[1]);
  }
}

// A single element of the stream (slow path: replacement columns only).
template <bool F32>
__device__ inline double philox_normal_at(uint64_t e, uint32_t stream, uint64_t seed) {
  double z[4];
  if (F32) {
    philox_normals<true>(e >> 2, stream, seed, z);
    return z[e & 3];
  }
  philox_normals<false>(e >> 1, stream, seed, z);
  return z[e & 1];
}

}  // namespace rsvd
