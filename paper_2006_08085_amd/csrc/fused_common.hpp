// Shared by the register-resident fused kernels: the compile-time neighbour
// patterns (ring, 2-D torus) and K rounds of Algorithm 3 on a column held in
// registers.
#pragma once

#include "detag_internal.h"
#include "dev_common.hpp"

namespace detag {
namespace fused {

constexpr int kThreads = 256;

// Workgroups are handed to the eight XCDs (each with its own L2) round-robin by their index.  Mapping index b
// to column tile (b % 8) * (tiles / 8) + b / 8 gives every XCD one contiguous eighth of the columns instead of
// every eighth tile, so the lines one L2 holds are neighbours in memory.  The tiles past a multiple of eight
// keep their own index.
__device__ __forceinline__ int64_t xcd_tile(uint32_t b, uint32_t tiles) {
  const uint32_t per = tiles / 8u;
  return b < per * 8u ? int64_t(b % 8u) * per + b / 8u : int64_t(b);
}

template <int N>
struct Ring {
  static constexpr int n = N, deg = 2;
  __host__ __device__ static constexpr int nb(int i, int k) { return k == 0 ? (i + N - 1) % N : (i + 1) % N; }
};

template <int R, int C>
struct Torus {
  static constexpr int n = R * C, deg = 4;
  __host__ __device__ static constexpr int nb(int i, int k) {
    const int r = i / C, c = i % C;
    return k == 0 ? ((r + R - 1) % R) * C + c
         : k == 1 ? ((r + 1) % R) * C + c
         : k == 2 ? r * C + (c + C - 1) % C
                  : r * C + (c + 1) % C;
  }
};

// The patterns the register-resident kernels are compiled for.  Calls f with a value of the pattern type that
// matches W (Ring<N> or Torus<R, C>) and returns its result; -1 if W is none of them.
template <class F>
int with_pattern(const HostW &W, F &&f) {
  if (W.structure == kRing) {
    switch (W.n) {
      case 4: return f(Ring<4>{});
      case 8: return f(Ring<8>{});
      case 12: return f(Ring<12>{});
      case 16: return f(Ring<16>{});
      case 24: return f(Ring<24>{});
      case 32: return f(Ring<32>{});
      case 48: return f(Ring<48>{});
      case 64: return f(Ring<64>{});
    }
  } else if (W.structure == kTorus) {
    if (W.trows == 8 && W.tcols == 8) return f(Torus<8, 8>{});
    if (W.trows == 4 && W.tcols == 4) return f(Torus<4, 4>{});
    if (W.trows == 4 && W.tcols == 8) return f(Torus<4, 8>{});
  }
  return -1;
}

// One round of Algorithm 3 in velocity form.  With v_r = z_r - z_{r-1} (v_0 = 0, since z_{-1} = z_0),
//   z_{r+1} = (1+eta) W^T z_r - eta z_{r-1}
// is the same as
//   v_{r+1,i} = b * sum_{j in nb(i)} (z_j - z_i) + eta * v_{r,i},   z_{r+1} = z_r + v_{r+1},   b = (1+eta)*w_nb
// (W_ii = 1 - deg*w_nb written out).  Two things make this the form to compute in fp32:
//  - a column whose workers all hold one value is a fixed point exactly, whatever the rounding of b and eta,
//    so the worker mean, which gradient tracking relies on, does not drift with the number of rounds;
//  - the only rounding at the magnitude of z is the final add; the recursion amplifies every rounding by up
//    to (1+(1+sqrt(eta))k) eta^(k/2) over the following k rounds, so fewer and smaller roundings matter
//    once eta is close to 1 (measured on 62 rounds at eta = 0.94: 2e-6 absolute against 1.3e-4 for
//    (1+eta)*(W_ii z_i + w_nb*sum) - eta*z_prev with separately rounded coefficients).
// Same operation count as that form (with the velocity kept divided by b, see ag_rounds).
struct Coef {
  float b, eta;
};

// sum of the neighbours' values, added pairwise so that deg equal values sum exactly
template <class T>
__device__ __forceinline__ float nb_sum(const float (&z)[T::n], int i) {
  static_assert(T::deg == 2 || T::deg == 4, "pairwise sum written for 2 or 4 neighbours");
  if constexpr (T::deg == 2) return z[T::nb(i, 0)] + z[T::nb(i, 1)];
  else return (z[T::nb(i, 0)] + z[T::nb(i, 1)]) + (z[T::nb(i, 2)] + z[T::nb(i, 3)]);
}

// sum_{j in nb(i)} (z_j - z_i)
template <class T>
__device__ __forceinline__ float lap(const float (&z)[T::n], int i) {
  return fmaf(-float(T::deg), z[i], nb_sum<T>(z, i));
}

// u <- eta * u + t as one three-operand instruction writing u's own register.  Left to the compiler, the
// loop-carried u becomes a two-operand v_fmac into t's register and a copy back: one instruction more per output
// and round, a seventh of the round loop.  The vector ALUs of these kernels are busy about two thirds of the time
// (counters), so the copy is not free everywhere, though on the machines where HBM sets the pace (3.9 ms for the
// gradient-fused step on the 8x8 torus at d = 11.2 M) taking it out measured no change.
__device__ __forceinline__ void momentum(float &u, float eta, float t) {
  asm("v_fma_f32 %0, %1, %0, %2" : "+v"(u) : "s"(eta), "v"(t));
}

// K >= 1 rounds starting from z_{-1} = z_0 = z.  Result in z; u is scratch: the velocity divided by b,
//   u_{r+1} = sum_nb (z_j - z_i) + eta * u_r,   z_{r+1} = z_r + b * u_{r+1},
// which is the recursion above with v = b*u and costs one multiplication less per output and round.
template <class T>
__device__ __forceinline__ void ag_rounds(float (&z)[T::n], float (&u)[T::n], const Coef &c, int K) {
#pragma unroll
  for (int i = 0; i < T::n; ++i) u[i] = lap<T>(z, i);
#pragma unroll
  for (int i = 0; i < T::n; ++i) z[i] = fmaf(c.b, u[i], z[i]);
  for (int r = 1; r < K; ++r) {
#pragma unroll
    for (int i = 0; i < T::n; ++i) momentum(u[i], c.eta, lap<T>(z, i));
#pragma unroll
    for (int i = 0; i < T::n; ++i) z[i] = fmaf(c.b, u[i], z[i]);
  }
}

// Register budget: the live state is 2 (gossip only) or 3 (phase) arrays of n
// floats per lane, plus the loads in flight.  The kernel asks for the matching
// waves-per-SIMD so the register allocator works against the real budget.
constexpr int waves_per_simd(int n, int mode) {
  const int need = n * (mode == 0 || mode == 3 ? 2 : 3) + 40;
  const int w = 512 / need;
  return w < 1 ? 1 : w > 8 ? 8 : w;
}

// Rows whose loads are in flight ahead of the row being consumed.  The loads
// of a tile are issued in row order through a software pipeline of this depth
// (the scheduling barriers pin that order); left alone, the compiler hoists all
// 4n loads of the tile to the top and spills.
// Measured on the 8x8 torus at d = 11.2 M: 4 to 15 rows ahead all give the same kernel time, 2 is 6 % slower.
constexpr int kRowsAhead = 12;

inline Coef make_coef(const HostW &W, float eta) {
  Coef c;
  c.b = float((1.0 + double(eta)) * W.w_nb);
  c.eta = eta;
  return c;
}

}  // namespace fused
}  // namespace detag
