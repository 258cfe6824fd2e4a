// Counter-based Gaussian noise on the device: Philox-4x32 with 10 rounds
// (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3",
// SC'11) followed by the Box-Muller transform.
//
// Noise of (step t, worker i, columns 4q..4q+3):
//   counter = (q mod 2^32, q div 2^32, i, t),  key = (seed mod 2^32, seed div 2^32)
//   u(r) = ((r >> 9) + 1/2) * 2^-23   (exact in fp32, never 0 or 1)
//   z0, z1 = sqrt(-2 ln u(r0)) * (cos, sin)(2 pi u(r1));  z2, z3 likewise from (r2, r3)
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace detag {

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t (&out)[4]) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r) k0 += W0, k1 += W1;
    const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
  }
  out[0] = c0, out[1] = c1, out[2] = c2, out[3] = c3;
}

__device__ __forceinline__ float unit_open(uint32_t r) { return (float(r >> 9) + 0.5f) * 0x1p-23f; }

__device__ __forceinline__ void box_muller(uint32_t ra, uint32_t rb, float &z0, float &z1) {
  const float rad = sqrtf(-2.0f * logf(unit_open(ra)));
  float s, c;
  sincospif(2.0f * unit_open(rb), &s, &c);
  z0 = rad * c;
  z1 = rad * s;
}

// The four standard normals of one Philox block.
__device__ __forceinline__ void normal4(uint64_t q, uint32_t worker, uint32_t step, uint32_t seed_lo, uint32_t seed_hi,
                                        float (&z)[4]) {
  uint32_t r[4];
  philox4x32_10(uint32_t(q & 0xffffffffu), uint32_t(q >> 32), worker, step, seed_lo, seed_hi, r);
  box_muller(r[0], r[1], z[0], z[1]);
  box_muller(r[2], r[3], z[2], z[3]);
}

}  // namespace detag
