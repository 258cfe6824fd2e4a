// K-round fused DeTAG phase for an arbitrary sparse gossip matrix with up to
// 256 workers and at most 8 neighbours per worker (e.g. a random regular graph
// with Metropolis weights).
//
// A block owns 64 columns and all n rows of them.  Wavefront w owns the rows
// w, w+4, w+8, ...; lane l owns column l.  Each lane keeps z_r and z_{r-1} of its
// own rows in registers; z_r of ALL rows also sits in LDS (rows x 64 fp32), where
// the neighbours of a row are read.  Row indices are wavefront-uniform and the
// neighbour lists have a fixed width, so they arrive through independent scalar
// loads the compiler can batch, and every LDS access is 64 consecutive words.
// One round = read the neighbours from LDS, barrier, write the new value back,
// barrier.  HBM sees the state once per phase (the ATC phase reads Y twice:
// 18 B instead of 16 B per element with bf16 state); the kernel is bound by LDS
// bandwidth, (deg+1) words per output per round.
//
// Paper: Algorithm 3 (accelerated gossip) and Algorithm 2 / the matrix form in
// the proof of Theorem 3 (phase update).
#include "dev_common.hpp"
#include "detag_internal.h"

namespace detag {
namespace {

constexpr int kThreads = 256, kWaves = 4, kCols = 64;

struct Ell {
  const int32_t *col;
  const float *val, *self;
};

// p <- (1+eta) * (w_self*z_own + sum_k w_k * lds[j_k]) - eta * p, for this lane's rows; then publish p.
template <int RPT, int DEG>
__device__ __forceinline__ void round_step(const float (&z)[RPT], float (&p)[RPT], float *lds, int w, int lane,
                                           const Ell &g, float cm, float neg_eta) {
#pragma unroll
  for (int r = 0; r < RPT; ++r) {
    const int s = w * RPT + r;
    float acc = g.self[s] * z[r];
#pragma unroll
    for (int k = 0; k < DEG; ++k) acc = fmaf(g.val[s * DEG + k], lds[g.col[s * DEG + k] * kCols + lane], acc);
    p[r] = fmaf(cm, acc, neg_eta * p[r]);
  }
  __syncthreads();  // every read of z_r is done
#pragma unroll
  for (int r = 0; r < RPT; ++r) lds[(w + kWaves * r) * kCols + lane] = p[r];
  __syncthreads();  // z_{r+1} is visible
}

template <int RPT>
__device__ __forceinline__ void publish(const float (&cur)[RPT], float *lds, int w, int lane) {
#pragma unroll
  for (int r = 0; r < RPT; ++r) lds[(w + kWaves * r) * kCols + lane] = cur[r];
  __syncthreads();
}

// K >= 1 rounds from z_{-1} = z_0 = cur.  Result in cur; prev is scratch.
template <int RPT, int DEG>
__device__ __forceinline__ void gossip(float (&cur)[RPT], float (&prev)[RPT], float *lds, int w, int lane,
                                       const Ell &g, float eta, int K) {
  const float cm = 1.f + eta, neg_eta = -eta;
  publish<RPT>(cur, lds, w, lane);
#pragma unroll
  for (int r = 0; r < RPT; ++r) prev[r] = cur[r];
  int r = 0;
  for (; r + 2 <= K; r += 2) {
    round_step<RPT, DEG>(cur, prev, lds, w, lane, g, cm, neg_eta);
    round_step<RPT, DEG>(prev, cur, lds, w, lane, g, cm, neg_eta);
  }
  if (r < K) {
    round_step<RPT, DEG>(cur, prev, lds, w, lane, g, cm, neg_eta);
#pragma unroll
    for (int q = 0; q < RPT; ++q) cur[q] = prev[q];
  }
}

// Window of row i of the tile; rows >= n get an empty window (loads give 0, stores are dropped).
template <typename E>
__device__ __forceinline__ rsrc_t win(const E *base, int64_t tile, int64_t ld, int i, int n, uint32_t valid) {
  return row_of(base, tile, ld, i < n ? i : 0, i < n ? valid : 0u);
}

// mode 0: Z <- M(Z) on X.  mode 1 (ATC): X <- M(X - alpha*Y), Y <- M(Y + Gn - Go).
// mode 2 (ALG2): X <- M(X) - alpha*M(Y), Y <- M(Y) + Gn - Go.
template <typename ST, int RPT, int DEG>
__global__ __launch_bounds__(kThreads, 2) void fused_generic_kernel(ST *X, ST *Y, const float *__restrict__ Gn,
                                                                    const float *__restrict__ Go, int n, int64_t d,
                                                                    int64_t ld, Ell g, float eta, float alpha, int K,
                                                                    int mode) {
  extern __shared__ float lds[];  // (4*RPT) x 64
  // the wavefront index is uniform: say so, or the row indices and with them every
  // neighbour-list access are treated as per-lane values
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int64_t tile = int64_t(blockIdx.x) * kCols;
  const uint32_t valid = uint32_t(d - tile < kCols ? d - tile : kCols);
  const uint32_t so = lane * uint32_t(sizeof(ST)), fo = lane * 4u;
  float cur[RPT], prev[RPT];
  if (mode == 0) {
#pragma unroll
    for (int r = 0; r < RPT; ++r) cur[r] = buf_load<ST>(win(X, tile, ld, w + kWaves * r, n, valid), so);
    gossip<RPT, DEG>(cur, prev, lds, w, lane, g, eta, K);
#pragma unroll
    for (int r = 0; r < RPT; ++r) buf_store<ST>(win(X, tile, ld, w + kWaves * r, n, valid), so, cur[r]);
  } else if (mode == 1) {
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
      const int i = w + kWaves * r;
      cur[r] = fmaf(-alpha, buf_load<ST>(win(Y, tile, ld, i, n, valid), so), buf_load<ST>(win(X, tile, ld, i, n, valid), so));
    }
    gossip<RPT, DEG>(cur, prev, lds, w, lane, g, eta, K);
#pragma unroll
    for (int r = 0; r < RPT; ++r) buf_store<ST>(win(X, tile, ld, w + kWaves * r, n, valid), so, cur[r]);
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
      const int i = w + kWaves * r;
      cur[r] = buf_load<ST>(win(Y, tile, ld, i, n, valid), so) + buf_load<float>(win(Gn, tile, ld, i, n, valid), fo) -
               buf_load<float>(win(Go, tile, ld, i, n, valid), fo);
    }
    gossip<RPT, DEG>(cur, prev, lds, w, lane, g, eta, K);
#pragma unroll
    for (int r = 0; r < RPT; ++r) buf_store<ST>(win(Y, tile, ld, w + kWaves * r, n, valid), so, cur[r]);
  } else {
    // M(Y) first: both outputs need it
#pragma unroll
    for (int r = 0; r < RPT; ++r) cur[r] = buf_load<ST>(win(Y, tile, ld, w + kWaves * r, n, valid), so);
    gossip<RPT, DEG>(cur, prev, lds, w, lane, g, eta, K);
    float v[RPT];
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
      v[r] = cur[r];
      cur[r] = buf_load<ST>(win(X, tile, ld, w + kWaves * r, n, valid), so);
    }
    gossip<RPT, DEG>(cur, prev, lds, w, lane, g, eta, K);
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

template <typename ST, int RPT, int DEG>
int launch_k(const Shape &s, const Ell &g, int mode, void *X, void *Y, const float *Gn, const float *Go, float alpha,
             int K, float eta, void *stream) {
  const dim3 grid(ceil_div_i64(s.d, kCols));
  const size_t lds_bytes = size_t(RPT) * kWaves * kCols * sizeof(float);  // rows padded to 4*RPT; 64 KiB at most
  fused_generic_kernel<ST, RPT, DEG><<<grid, kThreads, lds_bytes, static_cast<hipStream_t>(stream)>>>(
      static_cast<ST *>(X), static_cast<ST *>(Y), Gn, Go, s.n, s.d, s.ld, g, eta, alpha, K, mode);
  return hip_rc(hipGetLastError());
}

template <typename ST, int RPT>
int launch_r(const Shape &s, const Ell &g, int deg, int mode, void *X, void *Y, const float *Gn, const float *Go,
             float alpha, int K, float eta, void *stream) {
  switch (deg) {
    case 2: return launch_k<ST, RPT, 2>(s, g, mode, X, Y, Gn, Go, alpha, K, eta, stream);
    case 4: return launch_k<ST, RPT, 4>(s, g, mode, X, Y, Gn, Go, alpha, K, eta, stream);
    case 8: return launch_k<ST, RPT, 8>(s, g, mode, X, Y, Gn, Go, alpha, K, eta, stream);
  }
  return -1;
}

template <typename ST>
int launch_t(const Shape &s, const Ell &g, int rpt, int deg, int mode, void *X, void *Y, const float *Gn,
             const float *Go, float alpha, int K, float eta, void *stream) {
  switch (rpt) {
    case 16: return launch_r<ST, 16>(s, g, deg, mode, X, Y, Gn, Go, alpha, K, eta, stream);
    case 32: return launch_r<ST, 32>(s, g, deg, mode, X, Y, Gn, Go, alpha, K, eta, stream);
    case 64: return launch_r<ST, 64>(s, g, deg, mode, X, Y, Gn, Go, alpha, K, eta, stream);
  }
  return -1;
}

}  // namespace

bool build_ell(const HostW &W, EllHost &out) {
  const int n = W.n;
  if (n > 64 * kWaves) return false;
  int maxdeg = 0;
  for (int i = 0; i < n; ++i) {
    int cnt = 0;
    for (int k = W.rowptr[i]; k < W.rowptr[i + 1]; ++k) cnt += W.colidx[k] != i;
    maxdeg = cnt > maxdeg ? cnt : maxdeg;
  }
  if (maxdeg > 8) return false;
  out.deg = maxdeg <= 2 ? 2 : maxdeg <= 4 ? 4 : 8;
  out.rpt = n <= 16 * kWaves ? 16 : n <= 32 * kWaves ? 32 : 64;
  const int slots = out.rpt * kWaves;
  out.col.assign(size_t(slots) * out.deg, 0);
  out.val.assign(size_t(slots) * out.deg, 0.f);
  out.self.assign(slots, 0.f);
  for (int i = 0; i < n; ++i) {
    const int s = (i % kWaves) * out.rpt + i / kWaves;
    int k2 = 0;
    for (int k = W.rowptr[i]; k < W.rowptr[i + 1]; ++k) {
      if (W.colidx[k] == i) {
        out.self[s] = float(W.vals[k]);
      } else {
        out.col[size_t(s) * out.deg + k2] = W.colidx[k];
        out.val[size_t(s) * out.deg + k2] = float(W.vals[k]);
        ++k2;
      }
    }
    for (; k2 < out.deg; ++k2) out.col[size_t(s) * out.deg + k2] = i;  // weight 0, a valid row to read
  }
  return true;
}

bool fused_generic_available(const HostW &W, const Shape &) {
  EllHost e;
  return build_ell(W, e);
}

int launch_fused_generic(const Shape &s, const HostW &, const DevCsr &w, int mode, void *X, void *Y, const float *Gn,
                         const float *Go, float alpha, int K, float eta, void *stream) {
  if (K < 1 || !w.ell_col) return -1;
  Ell g{w.ell_col, w.ell_val, w.ell_self};
  return s.bf16 ? launch_t<bf16_t>(s, g, w.ell_rpt, w.ell_deg, mode, X, Y, Gn, Go, alpha, K, eta, stream)
                : launch_t<float>(s, g, w.ell_rpt, w.ell_deg, mode, X, Y, Gn, Go, alpha, K, eta, stream);
}

}  // namespace detag
