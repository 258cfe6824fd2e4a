// Gradient query and DeTAG phase in one pass, for the diagonal-quadratic
// objective on ring / 2-D torus gossip matrices:
//
//   G+ = h * (X - b) + sigma * z              (gradient query of Algorithm 2, at the phase-start model)
//   X+ = M(X - alpha*Y),  Y+ = M(Y + G+ - G)  (phase update, matrix form in the proof of Theorem 3)
// or, as Algorithm 2 prints it,  X+ = M(X) - alpha*M(Y),  Y+ = M(Y) + G+ - G
//
// with M the K-step accelerated gossip of Algorithm 3.  The gradient needs X,
// which the phase loads anyway, so fusing it saves one read of X, one write and
// one read of the gradient: per element the kernel reads X, Y, G, b and writes
// X, Y, G (28 B, fp32) where the two separate kernels move 36 B.  G is updated
// in place: row i of the old gradient is read just before the new one is stored.
//
// Same register-resident layout as the plain fused phase (one lane = one
// column, all n rows on chip; for 64 workers part of the tracker side waits in
// LDS, see kParkedRows).  The Gaussian noise is counter-based; one
// Philox block yields the four normals of four adjacent columns of one worker,
// so the four lanes of a quad each generate the block of one of four
// consecutive rows and exchange the results with two DPP quad permutes (a 4x4
// transpose): every lane evaluates one block per four rows instead of four.
#include "detag_internal.h"
#include "fused_common.hpp"
#include "noise_dev.hpp"

namespace detag {
namespace {

using namespace fused;

// Rows of the tracker side parked in LDS while the model side runs its rounds, for patterns of 64 workers.
// With all three arrays (u, v and the round scratch p) in registers a lane needs 192 + staging registers, two
// wavefronts per SIMD; with 48 of v's 64 rows in LDS (48 KiB per block, each lane reading back only what it
// wrote: no barrier) it needs 146, three wavefronts per SIMD and three blocks per compute unit, which hides
// more of the noise and round arithmetic under the other blocks' memory phases.
constexpr int kParkedRows = 48;
// HPW: the curvature h is an n x ld matrix (one row per worker, one more streamed array: 32 B per element) instead
// of one d-vector shared by all workers.
// Wavefronts per SIMD asked of the register allocator: three with the parked rows at 64 workers, else the phase
// kernels' figure, one less where all rows' loads of five arrays are in flight at once beside the three resident
// arrays (12 workers with per-worker curvature: 16 bytes of scratch per lane otherwise).
constexpr int quad_waves(int n, bool hpw) {
  return n >= 64 ? 3 : waves_per_simd(n, 1) - (hpw && n == 12 ? 1 : 0);
}

template <class T, typename ST, bool HPW>
__global__ __launch_bounds__(kThreads, quad_waves(T::n, HPW)) void fused_quadratic_kernel(
    ST *X, ST *Y, float *G, const float *__restrict__ h, const float *__restrict__ b, int64_t d, int64_t ld, Coef c,
    float alpha, int K, float sigma, uint32_t seed_lo, uint32_t seed_hi, uint32_t step) {
  constexpr int N = T::n;
  static_assert(N % 4 == 0, "rows are processed in groups of four");
  constexpr int NL = N >= 64 ? kParkedRows : 0;
  constexpr int NR = N - NL;
  constexpr int D = kRowsAhead < N ? kRowsAhead : N;
  __shared__ float vl[NL > 0 ? NL * kThreads : 1];
  const int64_t tile = xcd_tile(blockIdx.x, gridDim.x) * kThreads;
  const uint32_t valid = uint32_t(d - tile < kThreads ? d - tile : kThreads);
  const uint32_t so = threadIdx.x * uint32_t(sizeof(ST)), fo = threadIdx.x * 4u;
  const unsigned j = threadIdx.x & 3u;
  const uint64_t q = uint64_t(tile + threadIdx.x) >> 2;
  const float hc = HPW ? 0.f : buf_load<float>(make_rsrc(h + tile, valid * 4u), fo);
  float u[N], p[N], vr[NR > 0 ? NR : 1];
  float lx[N], ly[N], lg[N], lb[N], lh[HPW ? N : 1];
#pragma unroll
  for (int i = 0; i < D; ++i) {
    lx[i] = buf_load<ST>(row_of(X, tile, ld, i, valid), so);
    ly[i] = buf_load<ST>(row_of(Y, tile, ld, i, valid), so);
    lg[i] = buf_load<float>(row_of(G, tile, ld, i, valid), fo);
    lb[i] = buf_load<float>(row_of(b, tile, ld, i, valid), fo);
    if constexpr (HPW) lh[i] = buf_load<float>(row_of(h, tile, ld, i, valid), fo);
  }
  __builtin_amdgcn_sched_barrier(0);
  // All the noise of the tile is generated now, while the first rows' loads are in flight, and parked in p
  // (free until the rounds).  Generated inside the row loop instead, the Philox and Box-Muller arithmetic
  // spaces the loads out: fewer reads in flight, 2 % more kernel time on the 8x8 torus at d = 11.2 M.
  if (sigma != 0.f) {
#pragma unroll
    for (int i = 0; i < N; i += 4) {  // noise of rows i..i+3 at this lane's column
      float z[4];
      normal4(q, uint32_t(i) + j, step, seed_lo, seed_hi, z);
      quad_transpose(z, j);
      p[i] = z[0], p[i + 1] = z[1], p[i + 2] = z[2], p[i + 3] = z[3];
    }
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) p[i] = 0.f;
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (i + D < N) {
      lx[i + D] = buf_load<ST>(row_of(X, tile, ld, i + D, valid), so);
      ly[i + D] = buf_load<ST>(row_of(Y, tile, ld, i + D, valid), so);
      lg[i + D] = buf_load<float>(row_of(G, tile, ld, i + D, valid), fo);
      lb[i + D] = buf_load<float>(row_of(b, tile, ld, i + D, valid), fo);
      if constexpr (HPW) lh[i + D] = buf_load<float>(row_of(h, tile, ld, i + D, valid), fo);
    }
    const float g = fmaf(sigma, p[i], (HPW ? lh[i] : hc) * (lx[i] - lb[i]));
    u[i] = fmaf(-alpha, ly[i], lx[i]);
    float vi = ly[i] + g - lg[i];
    pin_vgpr(vi);
    if (i < NR) vr[i] = vi;
    else vl[(i - NR) * kThreads + threadIdx.x] = vi;
    buf_store<float>(row_of(G, tile, ld, i, valid), fo, g);
    __builtin_amdgcn_sched_barrier(0);
  }
  ag_rounds<T>(u, p, c, K);
  __builtin_amdgcn_sched_barrier(0);
  X = launder_uniform(X);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    buf_store<ST>(row_of(X, tile, ld, i, valid), so, u[i]);
    if (i < NR) u[i] = vr[i];
    else u[i] = vl[(i - NR) * kThreads + threadIdx.x];
  }
  __builtin_amdgcn_sched_barrier(0);
  ag_rounds<T>(u, p, c, K);
  __builtin_amdgcn_sched_barrier(0);
  Y = launder_uniform(Y);
#pragma unroll
  for (int i = 0; i < N; ++i) buf_store<ST>(row_of(Y, tile, ld, i, valid), so, u[i]);
}

// Algorithm 2 as printed: the gossip runs on X and Y themselves and the gradients enter after it,
//   G+ = h*(X - b) + sigma*z;  X+ = M(X) - alpha*M(Y);  Y+ = M(Y) + G+ - G.
// The new gradient has to outlive both runs of rounds, so the tile keeps four values per element: X, Y and the
// round scratch in registers, the gradient in LDS (n KiB per block; every lane reads back only what it wrote, so
// there is no barrier).  The old gradient is read at the end, row by row just ahead of the row's stores, and
// overwritten in place: the same 28 B per element (32 B with per-worker curvature) as the ATC form.
template <class T, typename ST, bool HPW>
__global__ __launch_bounds__(kThreads, waves_per_simd(T::n, 1)) void fused_quadratic_alg2_kernel(
    ST *X, ST *Y, float *G, const float *__restrict__ h, const float *__restrict__ b, int64_t d, int64_t ld, Coef c,
    float alpha, int K, float sigma, uint32_t seed_lo, uint32_t seed_hi, uint32_t step) {
  constexpr int N = T::n;
  static_assert(N % 4 == 0, "rows are processed in groups of four");
  constexpr int D = kRowsAhead < N ? kRowsAhead : N;
  __shared__ float gl[N * kThreads];
  const int64_t tile = xcd_tile(blockIdx.x, gridDim.x) * kThreads;
  const uint32_t valid = uint32_t(d - tile < kThreads ? d - tile : kThreads);
  const uint32_t so = threadIdx.x * uint32_t(sizeof(ST)), fo = threadIdx.x * 4u;
  const unsigned j = threadIdx.x & 3u;
  const uint64_t q = uint64_t(tile + threadIdx.x) >> 2;
  const float hc = HPW ? 0.f : buf_load<float>(make_rsrc(h + tile, valid * 4u), fo);
  float u[N], v[N], p[N];
  {
    float lx[N], ly[N], lb[N], lh[HPW ? N : 1];
#pragma unroll
    for (int i = 0; i < D; ++i) {
      lx[i] = buf_load<ST>(row_of(X, tile, ld, i, valid), so);
      ly[i] = buf_load<ST>(row_of(Y, tile, ld, i, valid), so);
      lb[i] = buf_load<float>(row_of(b, tile, ld, i, valid), fo);
      if constexpr (HPW) lh[i] = buf_load<float>(row_of(h, tile, ld, i, valid), fo);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (sigma != 0.f) {  // the tile's noise, generated while the first rows' loads are in flight
#pragma unroll
      for (int i = 0; i < N; i += 4) {
        float z[4];
        normal4(q, uint32_t(i) + j, step, seed_lo, seed_hi, z);
        quad_transpose(z, j);
        p[i] = z[0], p[i + 1] = z[1], p[i + 2] = z[2], p[i + 3] = z[3];
      }
    } else {
#pragma unroll
      for (int i = 0; i < N; ++i) p[i] = 0.f;
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < N; ++i) {
      if (i + D < N) {
        lx[i + D] = buf_load<ST>(row_of(X, tile, ld, i + D, valid), so);
        ly[i + D] = buf_load<ST>(row_of(Y, tile, ld, i + D, valid), so);
        lb[i + D] = buf_load<float>(row_of(b, tile, ld, i + D, valid), fo);
        if constexpr (HPW) lh[i + D] = buf_load<float>(row_of(h, tile, ld, i + D, valid), fo);
      }
      gl[i * kThreads + threadIdx.x] = fmaf(sigma, p[i], (HPW ? lh[i] : hc) * (lx[i] - lb[i]));
      u[i] = lx[i];
      v[i] = ly[i];
      pin_vgpr(v[i]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  ag_rounds<T>(v, p, c, K);
  __builtin_amdgcn_sched_barrier(0);
  ag_rounds<T>(u, p, c, K);
  __builtin_amdgcn_sched_barrier(0);
  X = launder_uniform(X), Y = launder_uniform(Y);
  float lgo[N];
#pragma unroll
  for (int i = 0; i < D; ++i) lgo[i] = buf_load<float>(row_of(G, tile, ld, i, valid), fo);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (i + D < N) lgo[i + D] = buf_load<float>(row_of(G, tile, ld, i + D, valid), fo);
    const float g = gl[i * kThreads + threadIdx.x];
    buf_store<ST>(row_of(X, tile, ld, i, valid), so, fmaf(-alpha, v[i], u[i]));
    buf_store<ST>(row_of(Y, tile, ld, i, valid), so, v[i] + g - lgo[i]);
    buf_store<float>(row_of(G, tile, ld, i, valid), fo, g);
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <class T>
int launch_s(const Shape &s, bool alg2, void *X, void *Y, float *G, const float *h, bool hpw, const float *b,
             const Coef &c, float alpha, int K, float sigma, uint64_t seed, uint32_t step, void *stream) {
  const dim3 grid(ceil_div_i64(s.d, kThreads));
  auto st = static_cast<hipStream_t>(stream);
  const uint32_t slo = uint32_t(seed & 0xffffffffu), shi = uint32_t(seed >> 32);
#define DETAG_QUAD(KERNEL, ST, HPW)                                                                              \
  KERNEL<T, ST, HPW><<<grid, kThreads, 0, st>>>(static_cast<ST *>(X), static_cast<ST *>(Y), G, h, b, s.d, s.ld, c, \
                                                alpha, K, sigma, slo, shi, step)
#define DETAG_QUAD_ST(KERNEL)                                                            \
  if (s.bf16) {                                                                          \
    if (hpw) DETAG_QUAD(KERNEL, bf16_t, true); else DETAG_QUAD(KERNEL, bf16_t, false);   \
  } else {                                                                               \
    if (hpw) DETAG_QUAD(KERNEL, float, true); else DETAG_QUAD(KERNEL, float, false);     \
  }
  if (alg2) { DETAG_QUAD_ST(fused_quadratic_alg2_kernel) } else { DETAG_QUAD_ST(fused_quadratic_kernel) }
#undef DETAG_QUAD_ST
#undef DETAG_QUAD
  return hip_rc(hipGetLastError());
}

}  // namespace

int launch_fused_quadratic(const Shape &s, const HostW &W, bool alg2, void *X, void *Y, float *G, const float *h,
                           bool h_per_worker, const float *b, float alpha, int K, float eta, float sigma, uint64_t seed,
                           uint32_t step, void *stream) {
  if (K < 1) return -1;
  const Coef c = make_coef(W, eta);
  return with_pattern(W, [&](auto t) {
    return launch_s<decltype(t)>(s, alg2, X, Y, G, h, h_per_worker, b, c, alpha, K, sigma, seed, step, stream);
  });
}

}  // namespace detag
