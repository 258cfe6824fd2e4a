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
    const uint64_t p0 = uint64_t(M0) * c0, p1 = uint64_t(M1) * c2;  // one 32x32->64 multiply each
    const uint32_t hi0 = uint32_t(p0 >> 32), lo0 = uint32_t(p0);
    const uint32_t hi1 = uint32_t(p1 >> 32), lo1 = uint32_t(p1);
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
  }
  out[0] = c0, out[1] = c1, out[2] = c2, out[3] = c3;
}

__device__ __forceinline__ float unit_open(uint32_t r) { return (float(r >> 9) + 0.5f) * 0x1p-23f; }

// The hardware's log2, sqrt and sin/cos (the last two take their argument in revolutions, which is what the
// transform needs) are used directly: over all 2^23 values u can take, sin and cos are within 1.3e-7
// (absolute) and the radius within 1.4e-7 (relative) of the exact values.
__device__ __forceinline__ void box_muller(uint32_t ra, uint32_t rb, float &z0, float &z1) {
  constexpr float kTwoLn2 = 1.3862943611198906f;  // -2 ln u = -(2 ln 2) log2 u
  const float rad = __builtin_amdgcn_sqrtf(-kTwoLn2 * __builtin_amdgcn_logf(unit_open(ra)));
  const float rev = unit_open(rb);
  z0 = rad * __builtin_amdgcn_cosf(rev);
  z1 = rad * __builtin_amdgcn_sinf(rev);
}

// The four standard normals of one Philox block.
__device__ __forceinline__ void normal4(uint64_t q, uint32_t worker, uint32_t step, uint32_t seed_lo, uint32_t seed_hi,
                                        float (&z)[4]) {
  uint32_t r[4];
  philox4x32_10(uint32_t(q & 0xffffffffu), uint32_t(q >> 32), worker, step, seed_lo, seed_hi, r);
  box_muller(r[0], r[1], z[0], z[1]);
  box_muller(r[2], r[3], z[2], z[3]);
}

// One Philox block yields the normals of four adjacent columns of one worker.  A kernel whose lanes own one
// column each and walk the rows four at a time lets the four lanes of a quad (four adjacent columns) generate
// the blocks of four consecutive rows, one each, and exchanges the results with two DPP quad permutes: a 4x4
// transpose, so that every lane evaluates one block per four rows instead of four.
template <int CTRL>
__device__ __forceinline__ float quad_perm(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// a[k] = M[j][k] in quad lane j  ->  a[k] = M[k][j]
__device__ __forceinline__ void quad_transpose(float (&a)[4], unsigned j) {
  const bool odd = j & 1u, hi = j & 2u;
  const float t0 = quad_perm<0xB1>(odd ? a[0] : a[1]);  // lanes j ^ 1
  const float t1 = quad_perm<0xB1>(odd ? a[2] : a[3]);
  const float c0 = odd ? t0 : a[0], c1 = odd ? a[1] : t0, c2 = odd ? t1 : a[2], c3 = odd ? a[3] : t1;
  const float s0 = quad_perm<0x4E>(hi ? c0 : c2);       // lanes j ^ 2
  const float s1 = quad_perm<0x4E>(hi ? c1 : c3);
  a[0] = hi ? s0 : c0, a[1] = hi ? s1 : c1, a[2] = hi ? c2 : s0, a[3] = hi ? c3 : s1;
}

}  // namespace detag
