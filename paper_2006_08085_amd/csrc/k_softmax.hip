// Mini-batch gradient of multinomial logistic regression, every worker on its
// own batch (the gradient query of Algorithm 2 for the label-sorted-shard
// workload).  Both contractions run on the bf16 matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulate):
//
//   logits[s,c] = sum_f feat[s,f] * Wt[c,f] + bias[c]        (B x F) . (F x C)
//   dW[c,f]     = sum_s delta[s,c] * feat[s,f]                (C x B) . (B x F)
//
// The features are bf16 data.  The fp32 operands (weights, softmax residuals
// delta) are split exactly into three bf16 terms w = hi + mid + lo; the three
// terms of class c sit in rows c, C+c, 2C+c of the 32-row MFMA tile (3C <= 32)
// and are summed after the contraction, so the products carry every bit of the
// fp32 operand and no rounding point has to be mirrored by a reference.
//
// MFMA 32x32x16 operand layout (lane l, m = l % 32, g = l / 32):
//   A: row m, k = 8g..8g+7      B: column m, k = 8g..8g+7
//   D: column m, register r -> row 8*(r/4) + 4g + r%4
#include "dev_common.hpp"
#include "detag_internal.h"

namespace detag {
namespace {

constexpr int kThreads = 256;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint16_t bf16_part(float w, int part) {
  // exact three-way split: w = hi + mid + lo, each a bf16
  const uint16_t hi = bf16_bits_rne(w);
  if (part == 0) return hi;
  const float r1 = w - __uint_as_float(uint32_t(hi) << 16);
  const uint16_t mid = bf16_bits_rne(r1);
  if (part == 1) return mid;
  const float r2 = r1 - __uint_as_float(uint32_t(mid) << 16);
  return bf16_bits_rne(r2);
}

__device__ __forceinline__ int d_row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

// grid (B/32, n).  One block = 32 samples of one worker; its 4 wavefronts split F.
__global__ __launch_bounds__(kThreads) void softmax_logits_kernel(int64_t ld, const float *__restrict__ X,
                                                                  const uint16_t *__restrict__ feat,
                                                                  const int32_t *__restrict__ labels,
                                                                  const int32_t *__restrict__ batch, int S, int F, int C,
                                                                  int B, float *__restrict__ delta,
                                                                  float *__restrict__ loss_part) {
  __shared__ float part[4][32][33];
  const int i = blockIdx.y, sb = blockIdx.x;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, m = lane & 31, g = lane >> 5;
  const bool row_ok = m < 3 * C;
  const int p = row_ok ? m / C : 0, c = row_ok ? m % C : 0;
  int idx = batch[int64_t(i) * B + sb * 32 + m];
  idx = idx < 0 ? 0 : idx >= S ? S - 1 : idx;
  const float *wrow = X + int64_t(i) * ld + int64_t(c) * F + 8 * g;
  const uint16_t *frow = feat + (int64_t(i) * S + idx) * F + 8 * g;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  for (int k0 = wave * 16; k0 < F; k0 += 64) {
    u16x8 a;
#pragma unroll
    for (int j = 0; j < 8; ++j) a[j] = row_ok ? bf16_part(wrow[k0 + j], p) : uint16_t(0);
    const u16x8 b = *reinterpret_cast<const u16x8 *>(frow + k0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0,
                                                  0, 0);
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) part[wave][d_row(r, g)][m] = acc[r];
  __syncthreads();
  if (threadIdx.x < 32) {
    const int s = sb * 32 + threadIdx.x;
    int y = labels[int64_t(i) * S + idx];  // idx is this lane's sample (m == threadIdx.x here)
    y = y < 0 ? 0 : y >= C ? C - 1 : y;
    const float *bias = X + int64_t(i) * ld + int64_t(C) * F;
    float logit[10];
    float mx = -3.0e38f;
#pragma unroll
    for (int cc = 0; cc < 10; ++cc) {
      float v = 0.f;
      if (cc < C) {
        for (int w = 0; w < 4; ++w) v += part[w][cc][threadIdx.x] + part[w][C + cc][threadIdx.x] + part[w][2 * C + cc][threadIdx.x];
        v += bias[cc];
        mx = fmaxf(mx, v);
      }
      logit[cc] = v;
    }
    float sum = 0.f;
#pragma unroll
    for (int cc = 0; cc < 10; ++cc)
      if (cc < C) {
        logit[cc] = expf(logit[cc] - mx);
        sum += logit[cc];
      }
    const float inv = 1.f / sum, invB = 1.f / float(B);
    float my_loss = 0.f;
#pragma unroll
    for (int cc = 0; cc < 10; ++cc)
      if (cc < C) {
        const float pr = logit[cc] * inv;
        if (cc == y) my_loss = -logf(pr);
        delta[(int64_t(i) * C + cc) * B + s] = (pr - (cc == y ? 1.f : 0.f)) * invB;
      }
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) my_loss += __shfl_down(my_loss, o, 64);
    if (threadIdx.x == 0) loss_part[int64_t(i) * (B / 32) + sb] = my_loss;
  }
}

// grid (ceil(F/128), n).  One wavefront = 32 feature columns of one worker; K runs over the B samples.
__global__ __launch_bounds__(kThreads) void softmax_grad_kernel(int64_t ld, const uint16_t *__restrict__ feat,
                                                                const int32_t *__restrict__ batch, int S, int F, int C,
                                                                int B, const float *__restrict__ delta,
                                                                const float *__restrict__ loss_part,
                                                                float *__restrict__ G, float *__restrict__ loss) {
  __shared__ float tile[4][32][33];
  const int i = blockIdx.y;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, m = lane & 31, g = lane >> 5;
  const int f0 = (blockIdx.x * 4 + wave) * 32;
  const bool cols_ok = f0 < F;  // F % 32 == 0: a wavefront's 32 columns are all in or all out
  const bool row_ok = m < 3 * C;
  const int p = row_ok ? m / C : 0, c = row_ok ? m % C : 0;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  if (cols_ok) {
    const float *drow = delta + (int64_t(i) * C + c) * B + 8 * g;
    const int32_t *brow = batch + int64_t(i) * B + 8 * g;
    for (int k0 = 0; k0 < B; k0 += 16) {
      u16x8 a, b;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        a[j] = row_ok ? bf16_part(drow[k0 + j], p) : uint16_t(0);
        int idx = brow[k0 + j];
        idx = idx < 0 ? 0 : idx >= S ? S - 1 : idx;
        b[j] = feat[(int64_t(i) * S + idx) * F + f0 + m];
      }
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc,
                                                    0, 0, 0);
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) tile[wave][d_row(r, g)][m] = acc[r];
  __syncthreads();
  if (cols_ok)
    for (int cc = g; cc < C; cc += 2)
      G[int64_t(i) * ld + int64_t(cc) * F + f0 + m] = tile[wave][cc][m] + tile[wave][C + cc][m] + tile[wave][2 * C + cc][m];
  if (blockIdx.x == 0) {
    if (threadIdx.x < C) {  // bias gradient: sum over the batch of delta (already divided by B)
      const float *dr = delta + (int64_t(i) * C + threadIdx.x) * B;
      float s = 0.f;
      for (int k = 0; k < B; ++k) s += dr[k];
      G[int64_t(i) * ld + int64_t(C) * F + threadIdx.x] = s;
    }
    if (threadIdx.x == 64 && loss) {
      float s = 0.f;
      for (int k = 0; k < B / 32; ++k) s += loss_part[int64_t(i) * (B / 32) + k];
      loss[i] = s / float(B);
    }
  }
}

}  // namespace

int64_t softmax_scratch_floats(int n, int C, int B) { return int64_t(n) * C * B + int64_t(n) * (B / 32); }

int launch_grad_softmax(const Shape &s, const void *X, const uint16_t *feat, const int32_t *labels,
                        const int32_t *batch, int S, int F, int C, int B, float *scratch, float *G, float *loss,
                        void *stream) {
  auto st = static_cast<hipStream_t>(stream);
  float *delta = scratch, *loss_part = scratch + int64_t(s.n) * C * B;
  softmax_logits_kernel<<<dim3(B / 32, s.n), kThreads, 0, st>>>(s.ld, static_cast<const float *>(X), feat, labels, batch,
                                                                S, F, C, B, delta, loss_part);
  int rc = hip_rc(hipGetLastError());
  if (rc) return rc;
  softmax_grad_kernel<<<dim3((F + 127) / 128, s.n), kThreads, 0, st>>>(s.ld, feat, batch, S, F, C, B, delta, loss_part, G,
                                                                       loss);
  return hip_rc(hipGetLastError());
}

}  // namespace detag
