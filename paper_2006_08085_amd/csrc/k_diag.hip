// Diagnostics: the worker mean (the output line of Algorithm 2) and the
// consensus distance ||X - 1 xbar^T||_F^2 bounded in the proof of Theorem 3.
// One lane owns one column and walks the n rows once; sums are kept in fp64 and
// taken relative to the first worker's value, so the distance stays meaningful
// when the workers almost agree.  Reductions use a
// fixed order (wavefront shuffle tree, then one block over the per-block
// partials): results are bit-reproducible.
#include "dev_common.hpp"
#include "detag_internal.h"

namespace detag {
namespace {

constexpr int kThreads = 256;

// X is read once per kernel: non-temporal.
__device__ __forceinline__ float stream_f32(const float *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ float stream_f32(const bf16_t *p) {
  return __uint_as_float(uint32_t(__builtin_nontemporal_load(&p->bits)) << 16);
}

template <typename ST>
__global__ __launch_bounds__(kThreads) void mean_kernel(int n, int64_t d, int64_t ld, const ST *__restrict__ X,
                                                        float *__restrict__ xbar) {
  const int64_t c = int64_t(blockIdx.x) * kThreads + threadIdx.x;
  if (c >= d) return;
  double s = 0.0;
#pragma unroll 16
  for (int i = 0; i < n; ++i) s += double(stream_f32(X + int64_t(i) * ld + c));  // 16 rows' loads in flight
  xbar[c] = float(s / n);
}

__device__ __forceinline__ double block_sum(double v) {
  __shared__ double part[kThreads / 64];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
  __syncthreads();
  double t = 0.0;
  if (threadIdx.x == 0)
    for (int w = 0; w < kThreads / 64; ++w) t += part[w];
  return t;  // valid in thread 0
}

template <typename ST>
__global__ __launch_bounds__(kThreads) void consensus_partial_kernel(int n, int64_t d, int64_t ld,
                                                                     const ST *__restrict__ X,
                                                                     double *__restrict__ partials) {
  const int64_t c = int64_t(blockIdx.x) * kThreads + threadIdx.x;
  double acc = 0.0;
  if (c < d) {
    // One pass: with e_i = x_i - x_0 (exact in fp64 for fp32 or bf16 inputs),
    //   sum_i (x_i - mean)^2 = sum_i e_i^2 - (sum_i e_i)^2 / n.
    // Both terms are of the size of the result (the shift by x_0 removes the common part of the column), so the
    // subtraction does not cancel, however close the workers are to agreement.
    const double x0 = double(stream_f32(X + c));
    double s1 = 0.0, s2 = 0.0;
#pragma unroll 16
    for (int i = 1; i < n; ++i) {
      const double e = double(stream_f32(X + int64_t(i) * ld + c)) - x0;
      s1 += e;
      s2 = fma(e, e, s2);
    }
    acc = s2 - s1 * s1 / n;
    acc = acc < 0.0 ? 0.0 : acc;
  }
  const double t = block_sum(acc);
  if (threadIdx.x == 0) partials[blockIdx.x] = t;
}

__global__ __launch_bounds__(kThreads) void sum_partials_kernel(int64_t count, const double *__restrict__ partials,
                                                                double *__restrict__ out) {
  // four independent sums per thread: one chain of dependent additions per thread leaves the block waiting on one
  // load at a time (42 us for the 43,648 partial sums of d = 11.2 M); the order of the additions is fixed
  double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
  int64_t k = threadIdx.x;
  for (; k + 3 * kThreads < count; k += 4 * kThreads) {
    a0 += partials[k], a1 += partials[k + kThreads], a2 += partials[k + 2 * kThreads], a3 += partials[k + 3 * kThreads];
  }
  for (; k < count; k += kThreads) a0 += partials[k];
  const double t = block_sum((a0 + a1) + (a2 + a3));
  if (threadIdx.x == 0) *out = t;
}

// Partial sums of detag_consensus_error_static: one slot per block of 256 columns.  The array is part of the
// library's code object, so every GPU the library runs on holds its own copy, at its own address, until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress; kernels receive the address
// that call returns.
__device__ __align__(256) double scratch[kStaticPartialsMax];

constexpr int kMaxDevices = 64;
double *g_scratch_ptr[kMaxDevices] = {};  // per device, set once by static_partials_init

}  // namespace

int static_partials_init(int device) {
  if (device < 0 || device >= kMaxDevices) return hip_rc(hipErrorInvalidDevice);
  if (g_scratch_ptr[device]) return 0;
  double *ptr = nullptr;
  const hipError_t e = hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch));
  if (e != hipSuccess) return hip_rc(e);
  g_scratch_ptr[device] = ptr;
  return 0;
}

double *static_partials(int device) {
  return device >= 0 && device < kMaxDevices ? g_scratch_ptr[device] : nullptr;
}

int launch_mean(const Shape &s, const void *X, float *xbar, void *stream) {
  const dim3 grid(ceil_div_i64(s.d, kThreads));
  auto st = static_cast<hipStream_t>(stream);
  if (s.bf16)
    mean_kernel<bf16_t><<<grid, kThreads, 0, st>>>(s.n, s.d, s.ld, static_cast<const bf16_t *>(X), xbar);
  else
    mean_kernel<float><<<grid, kThreads, 0, st>>>(s.n, s.d, s.ld, static_cast<const float *>(X), xbar);
  return hip_rc(hipGetLastError());
}

int64_t consensus_partials_count(const Shape &s) { return (s.d + kThreads - 1) / kThreads; }

int launch_consensus_error(const Shape &s, const void *X, double *partials, double *out, void *stream) {
  const int64_t blocks = consensus_partials_count(s);
  auto st = static_cast<hipStream_t>(stream);
  if (s.bf16)
    consensus_partial_kernel<bf16_t><<<dim3(blocks), kThreads, 0, st>>>(s.n, s.d, s.ld,
                                                                         static_cast<const bf16_t *>(X), partials);
  else
    consensus_partial_kernel<float><<<dim3(blocks), kThreads, 0, st>>>(s.n, s.d, s.ld,
                                                                        static_cast<const float *>(X), partials);
  int rc = hip_rc(hipGetLastError());
  if (rc) return rc;
  sum_partials_kernel<<<1, kThreads, 0, st>>>(blocks, partials, out);
  return hip_rc(hipGetLastError());
}

}  // namespace detag
