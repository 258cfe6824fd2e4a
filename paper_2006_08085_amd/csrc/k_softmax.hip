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
// Each fp32 operand is split once (the weights by a small kernel of their own,
// the residuals where they are produced) into bf16 arrays the contractions load
// directly: split inside the contraction loops, the same values were split by
// every block that used them, and that arithmetic was 40 % of the run time.
//
// MFMA 32x32x16 operand layout (lane l, m = l % 32, g = l / 32):
//   A: row m, k = 8g..8g+7      B: column m, k = 8g..8g+7
//   D: column m, register r -> row 8*(r/4) + 4g + r%4
#include "dev_common.hpp"
#include "detag_internal.h"

namespace detag {
namespace {

constexpr int kLogitWaves = 16, kLogitThreads = 64 * kLogitWaves;  // logits: 16 wavefronts split F
constexpr int kGradThreads = 256;                                  // weight gradient: 4 wavefronts x 32 columns
constexpr int kStage = 128;                                        // samples staged in LDS at a time
constexpr int kStagePitch = 136;                                   // bf16 per staged row: 272 B, 16-byte aligned,
                                                                   // and 8 rows apart land 32 banks apart

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

// Wsplit[i][p*C + c][f] = term p of X[i][c*F + f].  One thread = 8 consecutive f of one (i, c).
template <bool VEC>
__global__ __launch_bounds__(256) void softmax_split_kernel(int64_t ld, const float *__restrict__ X, int n, int F, int C,
                                                            uint16_t *__restrict__ wsplit) {
  const int64_t t = int64_t(blockIdx.x) * 256 + threadIdx.x;
  const int per_row = F / 8;
  if (t >= int64_t(n) * C * per_row) return;
  const int f = int(t % per_row) * 8, c = int((t / per_row) % C), i = int(t / (int64_t(per_row) * C));
  const float *src = X + int64_t(i) * ld + int64_t(c) * F + f;
  float v[8];
  if constexpr (VEC) {
    const float4 a = *reinterpret_cast<const float4 *>(src), b = *reinterpret_cast<const float4 *>(src + 4);
    v[0] = a.x, v[1] = a.y, v[2] = a.z, v[3] = a.w, v[4] = b.x, v[5] = b.y, v[6] = b.z, v[7] = b.w;
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = src[j];
  }
#pragma unroll
  for (int p = 0; p < 3; ++p) {
    u16x8 o;
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = bf16_part(v[j], p);
    *reinterpret_cast<u16x8 *>(wsplit + (int64_t(i) * 3 * C + p * C + c) * F + f) = o;
  }
}

// grid (B/32, n).  One block = 32 samples of one worker; its 16 wavefronts split F in steps of 16 features,
// six steps' operands in flight at a time.  Writes the residuals delta[i][c][s] = (p_c - y_c)/B in fp32 and
// their three bf16 terms dsplit[i][p*C + c][s].
__global__ __launch_bounds__(kLogitThreads) void softmax_logits_kernel(int64_t ld, const float *__restrict__ X,
                                                                       const uint16_t *__restrict__ wsplit,
                                                                       const uint16_t *__restrict__ feat,
                                                                       const int32_t *__restrict__ labels,
                                                                       const int32_t *__restrict__ batch, int S, int F,
                                                                       int C, int B, float *__restrict__ delta,
                                                                       uint16_t *__restrict__ dsplit,
                                                                       float *__restrict__ loss_part) {
  __shared__ float part[kLogitWaves][30][33];  // rows 3C <= 30 of every wavefront's tile
  const int i = blockIdx.y, sb = blockIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, m = lane & 31, g = lane >> 5;
  const bool row_ok = m < 3 * C;
  int idx = batch[int64_t(i) * B + sb * 32 + m];
  idx = idx < 0 ? 0 : idx >= S ? S - 1 : idx;
  const uint16_t *wrow = wsplit + (int64_t(i) * 3 * C + (row_ok ? m : 0)) * F + 8 * g;
  const uint16_t *frow = feat + (int64_t(i) * S + idx) * F + 8 * g;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  const int steps = F / 16;
  constexpr int U = 6;
  for (int ks = wave; ks < steps; ks += U * kLogitWaves) {
    u16x8 wv[U], fv[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ks + u * kLogitWaves < steps) {  // wavefront-uniform
        const int k0 = (ks + u * kLogitWaves) * 16;
        wv[u] = *reinterpret_cast<const u16x8 *>(wrow + k0);
        fv[u] = *reinterpret_cast<const u16x8 *>(frow + k0);
      }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (ks + u * kLogitWaves < steps) {
        if (!row_ok) wv[u] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};  // rows past 3C of the tile
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wv[u]),
                                                      __builtin_bit_cast(bf16x8, fv[u]), acc, 0, 0, 0);
      }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (d_row(r, g) < 30) part[wave][d_row(r, g)][m] = acc[r];
  __syncthreads();
  // logits[c][s] = bias[c] + the three split terms of class c summed over the wavefronts (fixed order):
  // one thread per (class, sample), result parked in wavefront 0's slice of `part`
  float lsum = 0.f;
  const int lc = threadIdx.x >> 5, ls = threadIdx.x & 31;
  if (lc < C) {
    for (int w = 0; w < kLogitWaves; ++w) lsum += part[w][lc][ls] + part[w][C + lc][ls] + part[w][2 * C + lc][ls];
    lsum += X[int64_t(i) * ld + int64_t(C) * F + lc];
  }
  __syncthreads();
  if (lc < C) part[0][lc][ls] = lsum;
  __syncthreads();
  if (threadIdx.x < 32) {
    const int s = sb * 32 + threadIdx.x;
    int y = labels[int64_t(i) * S + idx];  // idx is this lane's sample (m == threadIdx.x here)
    y = y < 0 ? 0 : y >= C ? C - 1 : y;
    float logit[10];
    float mx = -3.0e38f;
#pragma unroll
    for (int cc = 0; cc < 10; ++cc) {
      float v = 0.f;
      if (cc < C) {
        v = part[0][cc][threadIdx.x];
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
        const float dl = (pr - (cc == y ? 1.f : 0.f)) * invB;
        delta[(int64_t(i) * C + cc) * B + s] = dl;
#pragma unroll
        for (int pp = 0; pp < 3; ++pp) dsplit[(int64_t(i) * 3 * C + pp * C + cc) * B + s] = bf16_part(dl, pp);
      }
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) my_loss += __shfl_down(my_loss, o, 64);
    if (threadIdx.x == 0) loss_part[int64_t(i) * (B / 32) + sb] = my_loss;
  }
}

// grid (ceil(F/128), n).  One block = 128 feature columns of one worker, one wavefront = 32 of them; K runs
// over the B samples.  The batch's rows of those columns are gathered into LDS with 16-byte row loads (a
// sample's 128 columns are 256 contiguous bytes) and read back column-wise, 8 samples per lane, which is the
// operand layout the MFMA wants; reading them column-wise from memory would be 2-byte accesses.
__global__ __launch_bounds__(kGradThreads) void softmax_grad_kernel(int64_t ld, const uint16_t *__restrict__ feat,
                                                                    const int32_t *__restrict__ batch, int S, int F,
                                                                    int C, int B, const float *__restrict__ delta,
                                                                    const uint16_t *__restrict__ dsplit,
                                                                    const float *__restrict__ loss_part,
                                                                    float *__restrict__ G, float *__restrict__ loss) {
  __shared__ __attribute__((aligned(16))) uint16_t stage[kStage][kStagePitch];
  __shared__ float tile[4][30][33];
  const int i = blockIdx.y;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, m = lane & 31, g = lane >> 5;
  const int fc0 = blockIdx.x * 128, f0 = fc0 + wave * 32;
  const bool cols_ok = f0 < F;  // F % 32 == 0: a wavefront's 32 columns are all in or all out
  const bool row_ok = m < 3 * C;
  const int piece = threadIdx.x & 15, prow = threadIdx.x >> 4;  // staging: 16 pieces of 8 columns x 16 rows a pass
  const bool piece_ok = fc0 + 8 * piece < F;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  for (int s0 = 0; s0 < B; s0 += kStage) {
    const int ns = B - s0 < kStage ? B - s0 : kStage;  // a multiple of 32
    // this lane's residuals for every step of the stage, fetched together with the feature rows
    u16x8 dv[kStage / 16];
    const uint16_t *drow = dsplit + (int64_t(i) * 3 * C + (row_ok ? m : 0)) * B + s0 + 8 * g;
#pragma unroll
    for (int st = 0; st < kStage / 16; ++st)
      if (cols_ok && st * 16 < ns) dv[st] = *reinterpret_cast<const u16x8 *>(drow + st * 16);
    u16x8 rows[kStage / 16];
#pragma unroll
    for (int ps = 0; ps < kStage / 16; ++ps) {
      const int sr = ps * 16 + prow;
      if (sr < ns && piece_ok) {
        int idx = batch[int64_t(i) * B + s0 + sr];
        idx = idx < 0 ? 0 : idx >= S ? S - 1 : idx;
        rows[ps] = *reinterpret_cast<const u16x8 *>(feat + (int64_t(i) * S + idx) * F + fc0 + 8 * piece);
      }
    }
#pragma unroll
    for (int ps = 0; ps < kStage / 16; ++ps) {
      const int sr = ps * 16 + prow;
      if (sr < ns && piece_ok) *reinterpret_cast<u16x8 *>(&stage[sr][8 * piece]) = rows[ps];
    }
    __syncthreads();
    if (cols_ok) {
#pragma unroll
      for (int st = 0; st < kStage / 16; ++st)
        if (st * 16 < ns) {  // block-uniform
          u16x8 b;
#pragma unroll
          for (int j = 0; j < 8; ++j) b[j] = stage[st * 16 + 8 * g + j][wave * 32 + m];
          if (!row_ok) dv[st] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};  // rows past 3C of the tile
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, dv[st]),
                                                        __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
        }
    }
    __syncthreads();
  }
#pragma unroll
  for (int r = 0; r < 16; ++r)
    if (d_row(r, g) < 30) tile[wave][d_row(r, g)][m] = acc[r];
  __syncthreads();
  if (cols_ok)
    for (int cc = g; cc < C; cc += 2)
      G[int64_t(i) * ld + int64_t(cc) * F + f0 + m] = tile[wave][cc][m] + tile[wave][C + cc][m] + tile[wave][2 * C + cc][m];
  if (blockIdx.x == 0) {
    // bias gradient: sum over the batch of delta (already divided by B); wavefront w takes classes w, w+4, ...
    for (int cc = wave; cc < C; cc += 4) {
      const float *dr = delta + (int64_t(i) * C + cc) * B;
      float s = 0.f;
      for (int k = lane; k < B; k += 64) s += dr[k];
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o, 64);
      if (lane == 0) G[int64_t(i) * ld + int64_t(C) * F + cc] = s;
    }
    if (threadIdx.x == 64 && loss) {
      float s = 0.f;
      for (int k = 0; k < B / 32; ++k) s += loss_part[int64_t(i) * (B / 32) + k];
      loss[i] = s / float(B);
    }
  }
}

}  // namespace

namespace {
// scratch layout (floats): delta n*C*B | loss_part n*(B/32) rounded up to 4 | dsplit n*3C*B bf16 | wsplit n*3C*F bf16
int64_t round4(int64_t x) { return (x + 3) / 4 * 4; }
}  // namespace

int64_t softmax_scratch_floats(int n, int C, int B, int F) {
  return int64_t(n) * C * B + round4(int64_t(n) * (B / 32)) + int64_t(n) * 3 * C * B / 2 + int64_t(n) * 3 * C * F / 2;
}

int launch_grad_softmax(const Shape &s, const void *X, const uint16_t *feat, const int32_t *labels,
                        const int32_t *batch, int S, int F, int C, int B, float *scratch, float *G, float *loss,
                        void *stream) {
  auto st = static_cast<hipStream_t>(stream);
  float *delta = scratch, *loss_part = delta + int64_t(s.n) * C * B;
  uint16_t *dsplit = reinterpret_cast<uint16_t *>(loss_part + round4(int64_t(s.n) * (B / 32)));
  uint16_t *wsplit = dsplit + int64_t(s.n) * 3 * C * B;
  const float *x = static_cast<const float *>(X);
  // weight rows start at X + i*ld + c*F + 8k: 16-byte aligned iff X is and ld, F are multiples of 4
  const bool vec = s.ld % 4 == 0 && F % 4 == 0 && (reinterpret_cast<uintptr_t>(X) & 15) == 0;
  const int split_blocks = int((int64_t(s.n) * C * (F / 8) + 255) / 256);
  if (vec) softmax_split_kernel<true><<<split_blocks, 256, 0, st>>>(s.ld, x, s.n, F, C, wsplit);
  else softmax_split_kernel<false><<<split_blocks, 256, 0, st>>>(s.ld, x, s.n, F, C, wsplit);
  int rc = hip_rc(hipGetLastError());
  if (rc) return rc;
  softmax_logits_kernel<<<dim3(B / 32, s.n), kLogitThreads, 0, st>>>(s.ld, x, wsplit, feat, labels, batch, S, F, C, B,
                                                                     delta, dsplit, loss_part);
  rc = hip_rc(hipGetLastError());
  if (rc) return rc;
  softmax_grad_kernel<<<dim3((F + 127) / 128, s.n), kGradThreads, 0, st>>>(s.ld, feat, batch, S, F, C, B, delta, dsplit,
                                                                           loss_part, G, loss);
  return hip_rc(hipGetLastError());
}

}  // namespace detag
