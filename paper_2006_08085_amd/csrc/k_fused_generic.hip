// The LDS-resident kernels for an arbitrary sparse gossip matrix (layout and round arithmetic in
// fused_generic_common.hpp): plain K-round gossip and the two forms of the DeTAG phase, and the host side that
// packs the neighbour table.
//
// Paper: Algorithm 3 (accelerated gossip) and Algorithm 2 / the matrix form in
// the proof of Theorem 3 (phase update).
#include "fused_generic_common.hpp"

namespace detag {
namespace {

using namespace lds_tile;

// mode 0: Z <- M(Z) on X.  mode 1 (ATC): X <- M(X - alpha*Y), Y <- M(Y + Gn - Go).
// mode 2 (ALG2): X <- M(X) - alpha*M(Y), Y <- M(Y) + Gn - Go.
template <typename ST, int DEG, bool UNI, int MODE, int RPT>
__global__ __launch_bounds__(kThreads, 8) void fused_generic_kernel(ST *X, ST *Y, const float *__restrict__ Gn,
                                                                    const float *__restrict__ Go, int n, int64_t d,
                                                                    int64_t ld, const uint32_t *__restrict__ table,
                                                                    float eta, float alpha, int K) {
  extern __shared__ float lds[];  // 16*RPT x 64
  // the wavefront index is uniform: say so, or the row indices and with them every
  // table access are treated as per-lane values
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int64_t tile = int64_t(blockIdx.x) * kCols;
  const uint32_t valid = uint32_t(d - tile < kCols ? d - tile : kCols);
  const uint32_t so = lane * uint32_t(sizeof(ST)), fo = lane * 4u;
  constexpr int TS = table_stride(DEG, UNI);
  RowTab<DEG, UNI> tab[RPT];
#pragma unroll
  for (int r = 0; r < RPT; ++r)
#pragma unroll
    for (int q = 0; q < TS; ++q) tab[r].w[q] = table[(w * RPT + r) * TS + q];
  scale_uniform_weights<DEG, UNI, RPT>(tab, 1.f + eta);
  float cur[RPT], prev[RPT];
  auto row = [&](int r) { return w + kWaves * r; };
  // Loads and stores go four rows at a time with the scheduler fenced in between: left alone, the compiler
  // issues all 16 rows' loads of every array at once, and the registers they hold decide how many blocks
  // fit on a compute unit.  Two blocks per unit is what lets one block's memory phases run under the
  // other's rounds.
  constexpr int kBatch = RPT < 4 ? RPT : 4;
  if constexpr (MODE == 0) {
#pragma unroll
    for (int r0 = 0; r0 < RPT; r0 += kBatch) {
#pragma unroll
      for (int r = r0; r < r0 + kBatch; ++r) cur[r] = buf_load<ST>(win(X, tile, ld, row(r), n, valid), so);
      __builtin_amdgcn_sched_barrier(0);
    }
    gossip<DEG, UNI, RPT>(cur, prev, lds, w, lane, tab, eta, K);
#pragma unroll
    for (int r = 0; r < RPT; ++r) buf_store<ST>(win(X, tile, ld, row(r), n, valid), so, cur[r]);
  } else if constexpr (MODE == 1) {
    // every input is read once: the second gossip's input Y + Gn - Go waits in registers under the first
    float v0[RPT];
#pragma unroll
    for (int r0 = 0; r0 < RPT; r0 += kBatch) {
      float x[kBatch], y[kBatch], gn[kBatch], go[kBatch];
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        x[q] = buf_load<ST>(win(X, tile, ld, row(r0 + q), n, valid), so);
        y[q] = buf_load<ST>(win(Y, tile, ld, row(r0 + q), n, valid), so);
        gn[q] = buf_load<float>(win(Gn, tile, ld, row(r0 + q), n, valid), fo);
        go[q] = buf_load<float>(win(Go, tile, ld, row(r0 + q), n, valid), fo);
      }
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        cur[r0 + q] = fmaf(-alpha, y[q], x[q]);
        v0[r0 + q] = y[q] + gn[q] - go[q];
        pin_vgpr(v0[r0 + q]);  // the sum now, not its three operands carried through the rounds
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    gossip<DEG, UNI, RPT>(cur, prev, lds, w, lane, tab, eta, K);
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
      buf_store<ST>(win(X, tile, ld, row(r), n, valid), so, cur[r]);
      cur[r] = v0[r];
    }
    __builtin_amdgcn_sched_barrier(0);
    gossip<DEG, UNI, RPT>(cur, prev, lds, w, lane, tab, eta, K);
#pragma unroll
    for (int r = 0; r < RPT; ++r) buf_store<ST>(win(Y, tile, ld, row(r), n, valid), so, cur[r]);
  } else {
    // M(Y) first: both outputs need it
#pragma unroll
    for (int r0 = 0; r0 < RPT; r0 += kBatch) {
#pragma unroll
      for (int r = r0; r < r0 + kBatch; ++r) cur[r] = buf_load<ST>(win(Y, tile, ld, row(r), n, valid), so);
      __builtin_amdgcn_sched_barrier(0);
    }
    gossip<DEG, UNI, RPT>(cur, prev, lds, w, lane, tab, eta, K);
    float v[RPT];
#pragma unroll
    for (int r0 = 0; r0 < RPT; r0 += kBatch) {
#pragma unroll
      for (int r = r0; r < r0 + kBatch; ++r) {
        v[r] = cur[r];
        cur[r] = buf_load<ST>(win(X, tile, ld, row(r), n, valid), so);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    gossip<DEG, UNI, RPT>(cur, prev, lds, w, lane, tab, eta, K);
#pragma unroll
    for (int r0 = 0; r0 < RPT; r0 += kBatch) {
      float gn[kBatch], go[kBatch];
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        gn[q] = buf_load<float>(win(Gn, tile, ld, row(r0 + q), n, valid), fo);
        go[q] = buf_load<float>(win(Go, tile, ld, row(r0 + q), n, valid), fo);
      }
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        buf_store<ST>(win(X, tile, ld, row(r0 + q), n, valid), so, fmaf(-alpha, v[r0 + q], cur[r0 + q]));
        buf_store<ST>(win(Y, tile, ld, row(r0 + q), n, valid), so, v[r0 + q] + gn[q] - go[q]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}


template <typename ST, int DEG, bool UNI, int RPT>
int launch_r(const Shape &s, const uint32_t *table, int mode, void *X, void *Y, const float *Gn, const float *Go,
             float alpha, int K, float eta, void *stream) {
  const dim3 grid(ceil_div_i64(s.d, kCols));
  const size_t lds_bytes = size_t(kWaves) * RPT * kCols * sizeof(float);  // 4 KiB per row of a wavefront
  auto st = static_cast<hipStream_t>(stream);
  ST *x = static_cast<ST *>(X), *y = static_cast<ST *>(Y);
#define DETAG_MODE(M)                                                                                             \
  fused_generic_kernel<ST, DEG, UNI, M, RPT><<<grid, kThreads, lds_bytes, st>>>(x, y, Gn, Go, s.n, s.d, s.ld, table, \
                                                                                eta, alpha, K)
  switch (mode) {
    case 0: DETAG_MODE(0); break;
    case 1: DETAG_MODE(1); break;
    case 2: DETAG_MODE(2); break;
    default: return hip_rc(hipErrorInvalidValue);
  }
#undef DETAG_MODE
  return hip_rc(hipGetLastError());
}

template <typename ST, int DEG, bool UNI>
int launch_k(const Shape &s, const uint32_t *table, int mode, void *X, void *Y, const float *Gn, const float *Go,
             float alpha, int K, float eta, void *stream) {
#define DETAG_RPT(R) \
  case R: return launch_r<ST, DEG, UNI, R>(s, table, mode, X, Y, Gn, Go, alpha, K, eta, stream)
  switch (rows_per_wave(s.n)) {
    DETAG_RPT(1);
    DETAG_RPT(2);
    DETAG_RPT(4);
    DETAG_RPT(8);
    DETAG_RPT(16);
  }
#undef DETAG_RPT
  return -1;
}

template <typename ST>
int launch_t(const Shape &s, const uint32_t *table, int deg, bool uni, int mode, void *X, void *Y, const float *Gn,
             const float *Go, float alpha, int K, float eta, void *stream) {
#define DETAG_CASE(DG)                                                                                   \
  case DG:                                                                                               \
    return uni ? launch_k<ST, DG, true>(s, table, mode, X, Y, Gn, Go, alpha, K, eta, stream)              \
               : launch_k<ST, DG, false>(s, table, mode, X, Y, Gn, Go, alpha, K, eta, stream)
  switch (deg) {
    DETAG_CASE(2);
    DETAG_CASE(4);
    DETAG_CASE(8);
  }
#undef DETAG_CASE
  return -1;
}

uint32_t f32_bits(float f) {
  uint32_t u;
  static_assert(sizeof u == sizeof f, "");
  __builtin_memcpy(&u, &f, sizeof u);
  return u;
}

}  // namespace

bool build_ell(const HostW &W, EllHost &out) {
  const int n = W.n;
  if (n > kRowsMax) return false;
  int maxdeg = 0;
  bool uniform = true;
  for (int i = 0; i < n; ++i) {
    int cnt = 0;
    float first = 0.f;
    for (int k = W.rowptr[i]; k < W.rowptr[i + 1]; ++k) {
      if (W.colidx[k] == i) continue;
      const float v = float(W.vals[k]);
      if (cnt == 0) first = v;
      else if (v != first) uniform = false;
      ++cnt;
    }
    maxdeg = cnt > maxdeg ? cnt : maxdeg;
  }
  if (maxdeg > 8) return false;
  out.deg = maxdeg <= 2 ? 2 : maxdeg <= 4 ? 4 : 8;
  out.uniform = uniform;
  const int ts = table_stride(out.deg, uniform);
  const int rpt = rows_per_wave(n), slots = kWaves * rpt;
  out.table.assign(size_t(slots) * ts, 0u);
  for (int i = 0; i < slots; ++i) {
    uint32_t *t = &out.table[size_t((i % kWaves) * rpt + i / kWaves) * ts];
    const uint32_t own = uint32_t(i) * kCols * 4u;  // byte offset of row i in LDS (< 65536)
    uint32_t offs[8];
    float vals[8];
    for (int k = 0; k < 8; ++k) offs[k] = own, vals[k] = 0.f;  // padding: weight 0 (or a repeat, below), a valid row
    int cnt = 0;
    if (i < n)
      for (int k = W.rowptr[i]; k < W.rowptr[i + 1]; ++k)
        if (W.colidx[k] != i) offs[cnt] = uint32_t(W.colidx[k]) * kCols * 4u, vals[cnt] = float(W.vals[k]), ++cnt;
    for (int k = 0; k < out.deg; k += 2) t[k / 2] = offs[k] | (offs[k + 1] << 16);
    if (uniform) t[out.deg / 2] = f32_bits(vals[0]);  // one weight for the row; padded entries repeat the row itself
    else
      for (int k = 0; k < out.deg; ++k) t[out.deg / 2 + k] = f32_bits(vals[k]);
  }
  return true;
}

bool fused_generic_available(const HostW &W, const Shape &) {
  EllHost e;
  return build_ell(W, e);
}

int launch_fused_generic(const Shape &s, const HostW &, const DevCsr &w, int mode, void *X, void *Y, const float *Gn,
                         const float *Go, float alpha, int K, float eta, void *stream) {
  if (K < 1 || !w.ell_table) return -1;
  return s.bf16 ? launch_t<bf16_t>(s, w.ell_table, w.ell_deg, w.ell_uniform, mode, X, Y, Gn, Go, alpha, K, eta, stream)
                : launch_t<float>(s, w.ell_table, w.ell_deg, w.ell_uniform, mode, X, Y, Gn, Go, alpha, K, eta, stream);
}

}  // namespace detag
