// K-round fused DeTAG phase for an arbitrary sparse gossip matrix with up to
// 256 workers (e.g. a random regular graph with Metropolis weights).
//
// A block owns 64 columns and all n rows of them.  Wavefront w owns the rows
// w, w+4, w+8, ...; lane l owns column l.  Each lane keeps z_r and z_{r-1} of its
// own rows in registers; z_r of ALL rows also sits in LDS (rows x 64 fp32), where
// the neighbours of a row are read.  Row indices are wavefront-uniform, so the
// neighbour lists come through scalar loads and every LDS access is 64
// consecutive words.  One round = read deg neighbours from LDS, barrier, write
// the new value back, barrier.  HBM sees the state once per phase (the ATC phase
// reads Y twice: 18 B instead of 16 B per element with bf16 state); the kernel
// is bound by LDS bandwidth, (deg+1) words per output per round.
//
// Paper: Algorithm 3 (accelerated gossip) and Algorithm 2 / the matrix form in
// the proof of Theorem 3 (phase update).
#include "dev_common.hpp"
#include "detag_internal.h"

namespace detag {
namespace {

constexpr int kThreads = 256, kWaves = 4, kCols = 64;

struct Csr {
  const int32_t *rowptr, *colidx;
  const float *vals, *w_self;
};

// p <- (1+eta) * (w_self*z_own + sum_k w_k * lds[j_k]) - eta * p, for this lane's rows; then publish p.
template <int RPT>
__device__ __forceinline__ void round_step(const float (&z)[RPT], float (&p)[RPT], float *lds, int n, int w, int lane,
                                           const Csr &g, float cm, float neg_eta) {
#pragma unroll
  for (int r = 0; r < RPT; ++r) {
    const int i = w + kWaves * r;  // rows >= n are padding: empty list, zero self weight
    float acc = g.w_self[i] * z[r];
    const int k1 = g.rowptr[i + 1];
    for (int k = g.rowptr[i]; k < k1; ++k) acc = fmaf(g.vals[k], lds[g.colidx[k] * kCols + lane], acc);
    p[r] = fmaf(cm, acc, neg_eta * p[r]);
  }
  __syncthreads();  // every read of z_r is done
#pragma unroll
  for (int r = 0; r < RPT; ++r) {
    lds[(w + kWaves * r) * kCols + lane] = p[r];
  }
  __syncthreads();  // z_{r+1} is visible
}

// K >= 1 rounds from z_{-1} = z_0 = cur (already published in LDS).  Result in cur.
template <int RPT>
__device__ __forceinline__ void rounds(float (&cur)[RPT], float (&prev)[RPT], float *lds, int n, int w, int lane,
                                       const Csr &g, float eta, int K) {
  const float cm = 1.f + eta, neg_eta = -eta;
#pragma unroll
  for (int r = 0; r < RPT; ++r) prev[r] = cur[r];
  int r = 0;
  for (; r + 2 <= K; r += 2) {
    round_step<RPT>(cur, prev, lds, n, w, lane, g, cm, neg_eta);
    round_step<RPT>(prev, cur, lds, n, w, lane, g, cm, neg_eta);
  }
  if (r < K) {
    round_step<RPT>(cur, prev, lds, n, w, lane, g, cm, neg_eta);
#pragma unroll
    for (int q = 0; q < RPT; ++q) cur[q] = prev[q];
  }
}

template <int RPT>
__device__ __forceinline__ void publish(const float (&cur)[RPT], float *lds, int n, int w, int lane) {
#pragma unroll
  for (int r = 0; r < RPT; ++r) {
    lds[(w + kWaves * r) * kCols + lane] = cur[r];
  }
  __syncthreads();
}

// Window of row i of the tile; rows >= n get an empty window (loads give 0, stores are dropped).
template <typename E>
__device__ __forceinline__ rsrc_t win(const E *base, int64_t tile, int64_t ld, int i, int n, uint32_t valid) {
  return row_of(base, tile, ld, i < n ? i : 0, i < n ? valid : 0u);
}

// MODE 0: Z <- M(Z) on X.  MODE 1 (ATC): X <- M(X - alpha*Y), Y <- M(Y + Gn - Go).
// MODE 2 (ALG2): X <- M(X) - alpha*M(Y), Y <- M(Y) + Gn - Go.
template <typename ST, int RPT, int MODE>
__global__ __launch_bounds__(kThreads, 2) void fused_generic_kernel(ST *X, ST *Y, const float *__restrict__ Gn,
                                                                    const float *__restrict__ Go, int n, int64_t d,
                                                                    int64_t ld, Csr g, float eta, float alpha, int K) {
  extern __shared__ float lds[];  // (4*RPT) x 64
  // the wavefront index is uniform: say so, or the row indices and with them every
  // neighbour-list access are treated as per-lane values
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int64_t tile = int64_t(blockIdx.x) * kCols;
  const uint32_t valid = uint32_t(d - tile < kCols ? d - tile : kCols);
  const uint32_t so = lane * uint32_t(sizeof(ST)), fo = lane * 4u;
  float cur[RPT], prev[RPT];
  if constexpr (MODE == 0) {
#pragma unroll
    for (int r = 0; r < RPT; ++r) cur[r] = buf_load<ST>(win(X, tile, ld, w + kWaves * r, n, valid), so);
    publish<RPT>(cur, lds, n, w, lane);
    rounds<RPT>(cur, prev, lds, n, w, lane, g, eta, K);
#pragma unroll
    for (int r = 0; r < RPT; ++r) buf_store<ST>(win(X, tile, ld, w + kWaves * r, n, valid), so, cur[r]);
  } else if constexpr (MODE == 1) {
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
      const int i = w + kWaves * r;
      cur[r] = fmaf(-alpha, buf_load<ST>(win(Y, tile, ld, i, n, valid), so), buf_load<ST>(win(X, tile, ld, i, n, valid), so));
    }
    publish<RPT>(cur, lds, n, w, lane);
    rounds<RPT>(cur, prev, lds, n, w, lane, g, eta, K);
#pragma unroll
    for (int r = 0; r < RPT; ++r) buf_store<ST>(win(X, tile, ld, w + kWaves * r, n, valid), so, cur[r]);
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
      const int i = w + kWaves * r;
      cur[r] = buf_load<ST>(win(Y, tile, ld, i, n, valid), so) + buf_load<float>(win(Gn, tile, ld, i, n, valid), fo) -
               buf_load<float>(win(Go, tile, ld, i, n, valid), fo);
    }
    publish<RPT>(cur, lds, n, w, lane);
    rounds<RPT>(cur, prev, lds, n, w, lane, g, eta, K);
#pragma unroll
    for (int r = 0; r < RPT; ++r) buf_store<ST>(win(Y, tile, ld, w + kWaves * r, n, valid), so, cur[r]);
  } else {
    float v[RPT];
#pragma unroll
    for (int r = 0; r < RPT; ++r) v[r] = buf_load<ST>(win(Y, tile, ld, w + kWaves * r, n, valid), so);
    publish<RPT>(v, lds, n, w, lane);
    rounds<RPT>(v, prev, lds, n, w, lane, g, eta, K);
#pragma unroll
    for (int r = 0; r < RPT; ++r) cur[r] = buf_load<ST>(win(X, tile, ld, w + kWaves * r, n, valid), so);
    publish<RPT>(cur, lds, n, w, lane);
    rounds<RPT>(cur, prev, lds, n, w, lane, g, eta, K);
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
      const int i = w + kWaves * r;
      buf_store<ST>(win(X, tile, ld, i, n, valid), so, fmaf(-alpha, v[r], cur[r]));
      buf_store<ST>(win(Y, tile, ld, i, n, valid), so,
                    v[r] + buf_load<float>(win(Gn, tile, ld, i, n, valid), fo) -
                        buf_load<float>(win(Go, tile, ld, i, n, valid), fo));
    }
  }
}

template <typename ST, int RPT>
int launch_r(const Shape &s, const Csr &g, int mode, void *X, void *Y, const float *Gn, const float *Go, float alpha,
             int K, float eta, void *stream) {
  const dim3 grid(ceil_div_i64(s.d, kCols));
  const size_t lds_bytes = size_t(RPT) * kWaves * kCols * sizeof(float);  // rows padded to 4*RPT
  auto st = static_cast<hipStream_t>(stream);
  ST *x = static_cast<ST *>(X), *y = static_cast<ST *>(Y);
  switch (mode) {
    case 0: fused_generic_kernel<ST, RPT, 0><<<grid, kThreads, lds_bytes, st>>>(x, y, Gn, Go, s.n, s.d, s.ld, g, eta, alpha, K); break;
    case 1: fused_generic_kernel<ST, RPT, 1><<<grid, kThreads, lds_bytes, st>>>(x, y, Gn, Go, s.n, s.d, s.ld, g, eta, alpha, K); break;
    default: fused_generic_kernel<ST, RPT, 2><<<grid, kThreads, lds_bytes, st>>>(x, y, Gn, Go, s.n, s.d, s.ld, g, eta, alpha, K); break;
  }
  return hip_rc(hipGetLastError());
}

template <typename ST>
int launch_t(const Shape &s, const Csr &g, int mode, void *X, void *Y, const float *Gn, const float *Go, float alpha,
             int K, float eta, void *stream) {
  if (s.n <= 16 * kWaves) return launch_r<ST, 16>(s, g, mode, X, Y, Gn, Go, alpha, K, eta, stream);
  if (s.n <= 32 * kWaves) return launch_r<ST, 32>(s, g, mode, X, Y, Gn, Go, alpha, K, eta, stream);
  return launch_r<ST, 64>(s, g, mode, X, Y, Gn, Go, alpha, K, eta, stream);
}

}  // namespace

// (4*RPT) x 64 fp32 words of LDS: 64 KiB at n = 256, the default dynamic limit.  The neighbour-list
// arrays on the device are padded to 256 rows (empty lists, zero self weight).
bool fused_generic_available(const HostW &W, const Shape &) { return W.n <= 64 * kWaves; }

int launch_fused_generic(const Shape &s, const HostW &W, const DevCsr &w, int mode, void *X, void *Y, const float *Gn,
                         const float *Go, float alpha, int K, float eta, void *stream) {
  if (K < 1 || W.n > 64 * kWaves || !w.nb_rowptr) return -1;
  Csr g{w.nb_rowptr, w.nb_colidx, w.nb_vals, w.w_self};
  return s.bf16 ? launch_t<bf16_t>(s, g, mode, X, Y, Gn, Go, alpha, K, eta, stream)
                : launch_t<float>(s, g, mode, X, Y, Gn, Go, alpha, K, eta, stream);
}

}  // namespace detag
