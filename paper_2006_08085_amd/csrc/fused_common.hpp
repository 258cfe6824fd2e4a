// Shared by the register-resident fused kernels: the compile-time neighbour
// patterns (ring, 2-D torus) and K rounds of Algorithm 3 on a column held in
// registers.
#pragma once

#include "detag_internal.h"
#include "dev_common.hpp"

namespace detag {
namespace fused {

constexpr int kThreads = 256;

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

// Coefficients of one round: z_new = a*z_i + b*sum_nb z_j - eta*z_prev_i,
// a = (1+eta)*w_self, b = (1+eta)*w_nb.
struct Coef {
  float a, b, neg_eta, a_first;  // a_first = a - eta: first round, where z_prev = z
};

template <class T>
__device__ __forceinline__ float nb_sum(const float (&z)[T::n], int i) {
  float s = z[T::nb(i, 0)];
#pragma unroll
  for (int k = 1; k < T::deg; ++k) s += z[T::nb(i, k)];
  return s;
}

// p <- a*z + b*nbsum(z) - eta*p   (p holds z_{r-1} on entry and z_{r+1} on exit)
template <class T>
__device__ __forceinline__ void ag_round(const float (&z)[T::n], float (&p)[T::n], const Coef &c) {
#pragma unroll
  for (int i = 0; i < T::n; ++i) p[i] = fmaf(c.b, nb_sum<T>(z, i), fmaf(c.a, z[i], c.neg_eta * p[i]));
}

// K >= 1 rounds starting from z_{-1} = z_0 = u.  Result in u; p is scratch.
template <class T>
__device__ __forceinline__ void ag_rounds(float (&u)[T::n], float (&p)[T::n], const Coef &c, int K) {
#pragma unroll
  for (int i = 0; i < T::n; ++i) p[i] = fmaf(c.b, nb_sum<T>(u, i), c.a_first * u[i]);  // z_1 in p
  int r = 1;
  for (; r + 2 <= K; r += 2) {
    ag_round<T>(p, u, c);  // z_{r+1} in u
    ag_round<T>(u, p, c);  // z_{r+2} in p
  }
  if (r < K) {
    ag_round<T>(p, u, c);
  } else {
#pragma unroll
    for (int i = 0; i < T::n; ++i) u[i] = p[i];
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
#ifndef DETAG_ROWS_AHEAD
#define DETAG_ROWS_AHEAD 12
#endif
constexpr int kRowsAhead = DETAG_ROWS_AHEAD;

inline Coef make_coef(const HostW &W, float eta) {
  Coef c;
  c.a = float((1.0 + double(eta)) * W.w_self);
  c.b = float((1.0 + double(eta)) * W.w_nb);
  c.neg_eta = -eta;
  c.a_first = float((1.0 + double(eta)) * W.w_self - double(eta));
  return c;
}

}  // namespace fused
}  // namespace detag
