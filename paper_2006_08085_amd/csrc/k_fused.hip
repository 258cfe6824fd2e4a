// K-round fused DeTAG phase for ring and 2-D torus gossip matrices.
//
// Gossip mixes workers (rows) and never columns, so a set of columns together
// with ALL n rows is a closed system: one lane owns one column, keeps the n
// worker values of that column in registers, and runs all K rounds of
// Algorithm 3 there.  The neighbour pattern is a compile-time function of the
// row index, so every z[j] below is a fixed register.  HBM sees each state
// element once on the way in and once on the way out, whatever K is:
//   phase (ATC/ALG2): read X, Y, Gnew, Gold, write X, Y  = 24 B per element (fp32 state)
//   gossip only     : read Z, write Z                    =  8 B per element
// A wavefront reads 256 contiguous bytes of one row per load instruction and a
// 256-thread block 1 KiB; rows are n*ld apart, which the hardware sees as n
// (times four matrices) sequential streams.
//
// Paper: Algorithm 3 (accelerated gossip), Algorithm 2 (phase update) and the
// matrix form in the proof of Theorem 3.
#include "detag_internal.h"
#include "fused_common.hpp"

namespace detag {
namespace {

using namespace fused;


// MODE 0: Z <- M(Z) on X.  MODE 1 (ATC): X <- M(X - alpha*Y), Y <- M(Y + Gn - Go).
// MODE 2 (ALG2): X <- M(X) - alpha*M(Y), Y <- M(Y) + Gn - Go.
// MODE 3 (D-PSGD baseline of the Experiments section): X <- W^T X - alpha*Gn, one plain round (c built with eta = 0).
template <class T, typename ST, int MODE>
__global__ __launch_bounds__(kThreads, waves_per_simd(T::n, MODE)) void fused_structured_kernel(
    ST *X, ST *Y, const float *__restrict__ Gn, const float *__restrict__ Go, int64_t d, int64_t ld, Coef c,
    float alpha, int K) {
  constexpr int N = T::n;
  constexpr int D = kRowsAhead < N ? kRowsAhead : N;
  const int64_t tile = xcd_tile(blockIdx.x, gridDim.x) * kThreads;
  const uint32_t valid = uint32_t(d - tile < kThreads ? d - tile : kThreads);
  const uint32_t so = threadIdx.x * uint32_t(sizeof(ST));  // lane byte offset in a state row
  const uint32_t go4 = threadIdx.x * 4u;                   // ... in an fp32 row
  float u[N], p[N];
  if constexpr (MODE == 0) {
#pragma unroll
    for (int i = 0; i < N; ++i) u[i] = buf_load<ST>(row_of(X, tile, ld, i, valid), so);
    __builtin_amdgcn_sched_barrier(0);
    ag_rounds<T>(u, p, c, K);
    __builtin_amdgcn_sched_barrier(0);
    X = launder_uniform(X);
#pragma unroll
    for (int i = 0; i < N; ++i) buf_store<ST>(row_of(X, tile, ld, i, valid), so, u[i]);
  } else if constexpr (MODE == 3) {
#pragma unroll
    for (int i = 0; i < N; ++i) u[i] = buf_load<ST>(row_of(X, tile, ld, i, valid), so);
    __builtin_amdgcn_sched_barrier(0);
    X = launder_uniform(X);
    float lg[N];  // gradient rows arrive a few rows ahead of the stores that consume them
#pragma unroll
    for (int i = 0; i < D; ++i) lg[i] = buf_load<float>(row_of(Gn, tile, ld, i, valid), go4);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < N; ++i) {
      if (i + D < N) lg[i + D] = buf_load<float>(row_of(Gn, tile, ld, i + D, valid), go4);
      buf_store<ST>(row_of(X, tile, ld, i, valid), so, fmaf(-alpha, lg[i], fmaf(c.b, lap<T>(u, i), u[i])));
      __builtin_amdgcn_sched_barrier(0);
    }
  } else {
    static_assert(MODE == 1 || MODE == 2, "unknown mode");
    float v[N];
    if constexpr (MODE == 1) {
      float lx[N], ly[N], lgn[N], lgo[N];
#pragma unroll
      for (int i = 0; i < D; ++i) {
        lx[i] = buf_load<ST>(row_of(X, tile, ld, i, valid), so);
        ly[i] = buf_load<ST>(row_of(Y, tile, ld, i, valid), so);
        lgn[i] = buf_load<float>(row_of(Gn, tile, ld, i, valid), go4);
        lgo[i] = buf_load<float>(row_of(Go, tile, ld, i, valid), go4);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < N; ++i) {
        if (i + D < N) {
          lx[i + D] = buf_load<ST>(row_of(X, tile, ld, i + D, valid), so);
          ly[i + D] = buf_load<ST>(row_of(Y, tile, ld, i + D, valid), so);
          lgn[i + D] = buf_load<float>(row_of(Gn, tile, ld, i + D, valid), go4);
          lgo[i + D] = buf_load<float>(row_of(Go, tile, ld, i + D, valid), go4);
        }
        u[i] = fmaf(-alpha, ly[i], lx[i]);
        v[i] = ly[i] + lgn[i] - lgo[i];
        pin_vgpr(v[i]);
        __builtin_amdgcn_sched_barrier(0);
      }
      ag_rounds<T>(u, p, c, K);
      __builtin_amdgcn_sched_barrier(0);
      X = launder_uniform(X);
#pragma unroll
      for (int i = 0; i < N; ++i) buf_store<ST>(row_of(X, tile, ld, i, valid), so, u[i]);
      __builtin_amdgcn_sched_barrier(0);
      ag_rounds<T>(v, p, c, K);
      __builtin_amdgcn_sched_barrier(0);
      Y = launder_uniform(Y);
#pragma unroll
      for (int i = 0; i < N; ++i) buf_store<ST>(row_of(Y, tile, ld, i, valid), so, v[i]);
    } else {
#pragma unroll
      for (int i = 0; i < N; ++i) {
        u[i] = buf_load<ST>(row_of(X, tile, ld, i, valid), so);
        v[i] = buf_load<ST>(row_of(Y, tile, ld, i, valid), so);
      }
      __builtin_amdgcn_sched_barrier(0);
      ag_rounds<T>(v, p, c, K);
      __builtin_amdgcn_sched_barrier(0);
      ag_rounds<T>(u, p, c, K);
      __builtin_amdgcn_sched_barrier(0);
      // p is free now: the gradient rows are fetched a few rows ahead of the stores
      X = launder_uniform(X), Y = launder_uniform(Y);
      float lgn[N], lgo[N];
#pragma unroll
      for (int i = 0; i < D; ++i) {
        lgn[i] = buf_load<float>(row_of(Gn, tile, ld, i, valid), go4);
        lgo[i] = buf_load<float>(row_of(Go, tile, ld, i, valid), go4);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < N; ++i) {
        if (i + D < N) {
          lgn[i + D] = buf_load<float>(row_of(Gn, tile, ld, i + D, valid), go4);
          lgo[i + D] = buf_load<float>(row_of(Go, tile, ld, i + D, valid), go4);
        }
        buf_store<ST>(row_of(X, tile, ld, i, valid), so, fmaf(-alpha, v[i], u[i]));
        buf_store<ST>(row_of(Y, tile, ld, i, valid), so, v[i] + lgn[i] - lgo[i]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
}

// One round of Algorithm 3 with z_{r-1} given (one iteration of Algorithm 2's communication), for the patterns above:
//   out = z_r + b * sum_nb (z_j - z_i) + eta * (z_r - z_{r-1}),   b = (1+eta) * w_nb.
// All n rows of z_r in registers, z_{r-1} streamed a few rows ahead of the stores: 12 B per element (fp32), every row
// read once.  Every row of z_r is in registers before the first store and a row of z_{r-1} is read before the same
// row of out is written, so out may be z_{r-1} (the caller's usual choice) or z_r itself.
template <class T, typename ST>
__global__ __launch_bounds__(kThreads, waves_per_simd(T::n, 0)) void structured_round_kernel(
    const ST *cur, const ST *prev, ST *out, int64_t d, int64_t ld, Coef c) {
  constexpr int N = T::n;
  constexpr int D = kRowsAhead < N ? kRowsAhead : N;
  const int64_t tile = xcd_tile(blockIdx.x, gridDim.x) * kThreads;
  const uint32_t valid = uint32_t(d - tile < kThreads ? d - tile : kThreads);
  const uint32_t so = threadIdx.x * uint32_t(sizeof(ST));
  float u[N], lp[N];
#pragma unroll
  for (int i = 0; i < N; ++i) u[i] = buf_load<ST>(row_of(cur, tile, ld, i, valid), so);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < D; ++i) lp[i] = buf_load<ST>(row_of(prev, tile, ld, i, valid), so);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (i + D < N) lp[i + D] = buf_load<ST>(row_of(prev, tile, ld, i + D, valid), so);
    const float v = fmaf(c.eta, u[i] - lp[i], c.b * lap<T>(u, i));
    buf_store<ST>(row_of(out, tile, ld, i, valid), so, u[i] + v);
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <class T, typename ST>
int launch_t(const Shape &s, int mode, void *X, void *Y, const float *Gn, const float *Go, const Coef &c,
             float alpha, int K, void *stream) {
  const dim3 grid(ceil_div_i64(s.d, kThreads));
  auto st = static_cast<hipStream_t>(stream);
  ST *x = static_cast<ST *>(X), *y = static_cast<ST *>(Y);
  switch (mode) {
    case 0: fused_structured_kernel<T, ST, 0><<<grid, kThreads, 0, st>>>(x, y, Gn, Go, s.d, s.ld, c, alpha, K); break;
    case 1: fused_structured_kernel<T, ST, 1><<<grid, kThreads, 0, st>>>(x, y, Gn, Go, s.d, s.ld, c, alpha, K); break;
    case 3: fused_structured_kernel<T, ST, 3><<<grid, kThreads, 0, st>>>(x, y, Gn, Go, s.d, s.ld, c, alpha, K); break;
    default: fused_structured_kernel<T, ST, 2><<<grid, kThreads, 0, st>>>(x, y, Gn, Go, s.d, s.ld, c, alpha, K); break;
  }
  return hip_rc(hipGetLastError());
}

template <class T>
int launch_s(const Shape &s, int mode, void *X, void *Y, const float *Gn, const float *Go, const Coef &c,
             float alpha, int K, void *stream) {
  return s.bf16 ? launch_t<T, bf16_t>(s, mode, X, Y, Gn, Go, c, alpha, K, stream)
                : launch_t<T, float>(s, mode, X, Y, Gn, Go, c, alpha, K, stream);
}

}  // namespace

bool fused_structured_available(const HostW &W) {
  return with_pattern(W, [](auto) { return 0; }) == 0;
}

int launch_fused_structured(const Shape &s, const HostW &W, int mode, void *X, void *Y, const float *Gn,
                            const float *Go, float alpha, int K, float eta, void *stream) {
  if (K < 1) return -1;
  const Coef c = make_coef(W, eta);
  return with_pattern(W, [&](auto t) { return launch_s<decltype(t)>(s, mode, X, Y, Gn, Go, c, alpha, K, stream); });
}

int launch_structured_round(const Shape &s, const HostW &W, const void *cur, const void *prev, void *out, float eta,
                            void *stream) {
  const Coef c = make_coef(W, eta);
  const dim3 grid(ceil_div_i64(s.d, kThreads));
  auto st = static_cast<hipStream_t>(stream);
  return with_pattern(W, [&](auto t) {
    using T = decltype(t);
    if (s.bf16)
      structured_round_kernel<T, bf16_t><<<grid, kThreads, 0, st>>>(
          static_cast<const bf16_t *>(cur), static_cast<const bf16_t *>(prev), static_cast<bf16_t *>(out), s.d, s.ld, c);
    else
      structured_round_kernel<T, float><<<grid, kThreads, 0, st>>>(
          static_cast<const float *>(cur), static_cast<const float *>(prev), static_cast<float *>(out), s.d, s.ld, c);
    return hip_rc(hipGetLastError());
  });
}

}  // namespace detag
