// Local stochastic gradients of the synthetic objectives: the gradient query
// of Algorithm 2, every worker at its own model.
//
//   diagonal quadratic: G = h * (x - b_i) + sigma * z, z standard normal, either
//     read from an array or regenerated from the counter (seed, step, worker,
//     column) with Philox-4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) and the
//     Box-Muller transform.  A thread owns the four columns of one Philox block.
//   least squares: G_i = A_i^T (A_i x_i - b_i), two small passes.
#include "detag_internal.h"
#include "dev_common.hpp"
#include "noise_dev.hpp"

namespace detag {
namespace {

constexpr int kThreads = 256;
typedef float vf4_t __attribute__((ext_vector_type(4)));
typedef uint32_t vu2_t __attribute__((ext_vector_type(2)));

// A block works on kGradRows consecutive worker rows of its 1024 columns, so that a shared curvature vector is
// read once per kGradRows rows instead of once per row (read per row it is a fourth stream: measured 1.33 x the
// bytes of X, b and G on 64 x 11.2 M).
constexpr int kGradRows = 4;

template <typename ST, bool VEC>
__global__ __launch_bounds__(kThreads) void grad_quadratic_kernel(int n, int64_t d, int64_t ld, const ST *__restrict__ X,
                                                                  const float *__restrict__ h, int64_t h_row_stride,
                                                                  const float *__restrict__ b,
                                                                  const float *__restrict__ noise, float sigma,
                                                                  uint32_t seed_lo, uint32_t seed_hi, uint32_t step,
                                                                  float *__restrict__ G) {
  const int64_t q = int64_t(blockIdx.x) * kThreads + threadIdx.x;  // Philox block = 4 columns
  const int64_t c0 = q * 4;
  if (c0 >= d) return;
  const int i0 = blockIdx.y * kGradRows;
  const int valid = int(d - c0 < 4 ? d - c0 : 4);
  const bool wide = VEC && valid == 4;
  float hs[4] = {0.f, 0.f, 0.f, 0.f};
  if (h_row_stride == 0) {  // shared by the workers: read once, cached (other blocks read it too)
    if (wide) {
      const float4 th = *reinterpret_cast<const float4 *>(h + c0);
      hs[0] = th.x, hs[1] = th.y, hs[2] = th.z, hs[3] = th.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) hs[e] = e < valid ? h[c0 + e] : 0.f;
    }
  }
#pragma unroll
  for (int r = 0; r < kGradRows; ++r) {
    const int i = i0 + r;
    if (i >= n) break;
    const int64_t off = int64_t(i) * ld + c0;
    float x[4], hv[4], bv[4], z[4] = {0.f, 0.f, 0.f, 0.f};
    if (wide) {
      // X, b, the noise array, per-worker curvature and G are touched once: non-temporal
      if constexpr (sizeof(ST) == 4) {
        const vf4_t t = __builtin_nontemporal_load(reinterpret_cast<const vf4_t *>(X + off));
        x[0] = t.x, x[1] = t.y, x[2] = t.z, x[3] = t.w;
      } else {
        const vu2_t t = __builtin_nontemporal_load(reinterpret_cast<const vu2_t *>(X + off));
        x[0] = __uint_as_float(t.x << 16), x[1] = __uint_as_float(t.x & 0xffff0000u);
        x[2] = __uint_as_float(t.y << 16), x[3] = __uint_as_float(t.y & 0xffff0000u);
      }
      const vf4_t tb = __builtin_nontemporal_load(reinterpret_cast<const vf4_t *>(b + off));
      bv[0] = tb.x, bv[1] = tb.y, bv[2] = tb.z, bv[3] = tb.w;
      if (h_row_stride) {
        const vf4_t th = __builtin_nontemporal_load(reinterpret_cast<const vf4_t *>(h + int64_t(i) * h_row_stride + c0));
        hv[0] = th.x, hv[1] = th.y, hv[2] = th.z, hv[3] = th.w;
      }
      if (noise) {
        const vf4_t tz = __builtin_nontemporal_load(reinterpret_cast<const vf4_t *>(noise + off));
        z[0] = tz.x, z[1] = tz.y, z[2] = tz.z, z[3] = tz.w;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool ok = e < valid;
        x[e] = ok ? to_f32(X[off + e]) : 0.f;
        if (h_row_stride) hv[e] = ok ? h[int64_t(i) * h_row_stride + c0 + e] : 0.f;
        bv[e] = ok ? b[off + e] : 0.f;
        if (noise) z[e] = ok ? noise[off + e] : 0.f;
      }
    }
    if (!h_row_stride) {
#pragma unroll
      for (int e = 0; e < 4; ++e) hv[e] = hs[e];
    }
    if (!noise && sigma != 0.f) normal4(uint64_t(q), uint32_t(i), step, seed_lo, seed_hi, z);
    float g[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) g[e] = fmaf(sigma, z[e], hv[e] * (x[e] - bv[e]));
    if (wide) {
      const vf4_t tg = {g[0], g[1], g[2], g[3]};
      __builtin_nontemporal_store(tg, reinterpret_cast<vf4_t *>(G + off));
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (e < valid) G[off + e] = g[e];
    }
  }
}

// resid[i*m + r] = A_i[r,:] . x_i - b_i[r]; one wavefront per (i, r).
template <typename ST>
__global__ __launch_bounds__(kThreads) void lstsq_resid_kernel(int n, int m, int64_t d, int64_t ld,
                                                               const ST *__restrict__ X, const float *__restrict__ A,
                                                               const float *__restrict__ b,
                                                               float *__restrict__ resid) {
  const int64_t row = int64_t(blockIdx.x) * (kThreads / 64) + (threadIdx.x >> 6);  // = i*m + r
  if (row >= int64_t(n) * m) return;
  const int i = int(row / m);
  const int lane = threadIdx.x & 63;
  const float *a = A + row * d;
  const ST *x = X + int64_t(i) * ld;
  float acc = 0.f;
  for (int64_t c = lane; c < d; c += 64) acc = fmaf(a[c], to_f32(x[c]), acc);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o, 64);
  if (lane == 0) resid[row] = acc - b[row];
}

// G[i,c] = sum_r A_i[r,c] * resid[i,r]; one lane per column.
__global__ __launch_bounds__(kThreads) void lstsq_grad_kernel(int m, int64_t d, int64_t ld,
                                                              const float *__restrict__ A,
                                                              const float *__restrict__ resid,
                                                              float *__restrict__ G) {
  const int64_t c = int64_t(blockIdx.x) * kThreads + threadIdx.x;
  if (c >= d) return;
  const int i = blockIdx.y;
  const float *a = A + int64_t(i) * m * d + c;
  const float *r = resid + int64_t(i) * m;
  float acc = 0.f;
  for (int k = 0; k < m; ++k) acc = fmaf(a[int64_t(k) * d], r[k], acc);
  G[int64_t(i) * ld + c] = acc;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

int launch_grad_quadratic(const Shape &s, const void *X, const float *h, int h_per_worker, const float *b,
                          const float *noise, float sigma, uint64_t seed, uint32_t step, float *G, void *stream) {
  const int64_t blocks4 = (s.d + 3) / 4;
  const dim3 grid(ceil_div_i64(blocks4, kThreads), (s.n + kGradRows - 1) / kGradRows);
  auto st = static_cast<hipStream_t>(stream);
  const int64_t hstride = h_per_worker ? s.ld : 0;
  const bool vec = s.ld % 4 == 0 && aligned16(h) && aligned16(b) && aligned16(G) && (!noise || aligned16(noise)) &&
                   (reinterpret_cast<uintptr_t>(X) & (s.bf16 ? 7 : 15)) == 0;
  const uint32_t slo = uint32_t(seed & 0xffffffffu), shi = uint32_t(seed >> 32);
#define DETAG_LAUNCH(ST, V)                                                                                     \
  grad_quadratic_kernel<ST, V><<<grid, kThreads, 0, st>>>(s.n, s.d, s.ld, static_cast<const ST *>(X), h, hstride, b, \
                                                          noise, sigma, slo, shi, step, G)
  if (s.bf16) {
    if (vec) DETAG_LAUNCH(bf16_t, true); else DETAG_LAUNCH(bf16_t, false);
  } else {
    if (vec) DETAG_LAUNCH(float, true); else DETAG_LAUNCH(float, false);
  }
#undef DETAG_LAUNCH
  return hip_rc(hipGetLastError());
}

int launch_grad_lstsq(const Shape &s, const void *X, const float *A, const float *b, int m, float *resid, float *G,
                      void *stream) {
  auto st = static_cast<hipStream_t>(stream);
  const int64_t rows = int64_t(s.n) * m;
  const dim3 g1(ceil_div_i64(rows, kThreads / 64));
  if (s.bf16)
    lstsq_resid_kernel<bf16_t><<<g1, kThreads, 0, st>>>(s.n, m, s.d, s.ld, static_cast<const bf16_t *>(X), A, b, resid);
  else
    lstsq_resid_kernel<float><<<g1, kThreads, 0, st>>>(s.n, m, s.d, s.ld, static_cast<const float *>(X), A, b, resid);
  int rc = hip_rc(hipGetLastError());
  if (rc) return rc;
  lstsq_grad_kernel<<<dim3(ceil_div_i64(s.d, kThreads), s.n), kThreads, 0, st>>>(m, s.d, s.ld, A, resid, G);
  return hip_rc(hipGetLastError());
}

}  // namespace detag
