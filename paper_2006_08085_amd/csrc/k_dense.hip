// K rounds of accelerated gossip as one dense product on the matrix cores.
//
// Algorithm 3 of the paper is linear in its input: z_K = P z_0 with the matrix
// polynomial P = p_K(W^T), p_{k+1}(M) = (1+eta) M p_k(M) - eta p_{k-1}(M),
// p_0 = p_{-1} = I (the Chebyshev-like polynomial its analysis is about).  The
// host evaluates P once per (K, eta) in fp64; a phase of Algorithm 2 on n <= 256
// workers is then, for every column of the state, a 256 x 256 matrix-vector
// product: a dense contraction whose cost does not depend on K or on the degree
// of the graph, where the round-by-round kernel for arbitrary W is bound by LDS
// traffic that grows with both.
//
// v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  Operands are split into bf16
// terms whose sum is the fp32 value (P: hi + mid + lo on the host; the staged
// inputs on the device), and the products that matter at the state's precision
// are accumulated: for fp32 state 3 + 3 terms, the 6 products down to 2^-24;
// for bf16 state 2 + 2 terms and 3 products (a bf16 input is its own first term).
//
// One block = 64 columns, 4 wavefronts.  Staging: lane = column, a wavefront
// loads 8 consecutive rows (coalesced row segments), applies the phase's
// elementwise part (X - alpha Y, Y + Gnew - Gold), splits, and writes one 16-byte
// word per term to LDS laid out [term][column][row] -- exactly the B operand
// (column m, k = 8g..8g+7) of the MFMA.  Product: wavefront w owns output rows
// 64w..64w+63 (two 32-row tiles) of both 32-column tiles; the A operand comes
// from a copy of P the host pre-arranged in fragment order (one 1 KiB coalesced
// load per tile and k-step, served by L2).  MFMA operand layout (lane l,
// m = l % 32, g = l / 32):  A: row m, k = 8g..8g+7;  B: column m, k = 8g..8g+7;
// D: column m, register r -> row 8*(r/4) + 4g + r%4.
#include "detag_internal.h"
#include "dev_common.hpp"

namespace detag {
namespace {

constexpr int kCols = 64, kThreads = 256, kWaves = 4;
constexpr int kRowsMax = 256, kMTiles = kRowsMax / 32, kKSteps = kRowsMax / 16;
constexpr int kPitch = kRowsMax + 8;            // bf16 per staged column: 528 B, so that 16 columns hit 64 banks
constexpr int kTermElems = kCols * kPitch;      // one term of the staged tile

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ int d_row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

// v = t[0] + t[1] (+ t[2]) with bf16 terms, exact for three terms.
template <int T>
__device__ __forceinline__ void split_terms(float v, uint16_t (&t)[T]) {
  t[0] = bf16_bits_rne(v);
  if constexpr (T > 1) {
    const float r1 = v - __uint_as_float(uint32_t(t[0]) << 16);
    t[1] = bf16_bits_rne(r1);
    if constexpr (T > 2) t[2] = bf16_bits_rne(r1 - __uint_as_float(uint32_t(t[1]) << 16));
  }
}

// What is multiplied by P in a pass.
enum Pre : int { kPreX = 0, kPreXminusAlphaY = 1, kPreTrack = 2, kPreY = 3 };

// Rows 8q..8q+7 of the block's 64 columns -> the elementwise part -> TU bf16 terms in LDS.  Rows >= n are staged
// as zeros (their resource has no valid bytes).
template <typename ST, int TU, int PRE>
__device__ __forceinline__ void stage_rows(uint16_t *stage, int q, int lane, const ST *X, const ST *Y, const float *Gn,
                                           const float *Go, int n, int64_t tile, int64_t ld, uint32_t valid,
                                           float alpha) {
  const uint32_t so = lane * uint32_t(sizeof(ST)), fo = lane * 4u;
  float v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int row = 8 * q + e;
    const uint32_t ok = row < n ? valid : 0u;
    const int rr = row < n ? row : 0;
    if constexpr (PRE == kPreX) {
      v[e] = buf_load<ST>(row_of(X, tile, ld, rr, ok), so);
    } else if constexpr (PRE == kPreY) {
      v[e] = buf_load<ST>(row_of(Y, tile, ld, rr, ok), so);
    } else if constexpr (PRE == kPreXminusAlphaY) {
      const float x = buf_load<ST>(row_of(X, tile, ld, rr, ok), so), y = buf_load<ST>(row_of(Y, tile, ld, rr, ok), so);
      v[e] = fmaf(-alpha, y, x);
    } else {
      const float y = buf_load<ST>(row_of(Y, tile, ld, rr, ok), so);
      const float gn = buf_load<float>(row_of(Gn, tile, ld, rr, ok), fo), go = buf_load<float>(row_of(Go, tile, ld, rr, ok), fo);
      v[e] = y + gn - go;
    }
  }
  u16x8 o[TU];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    uint16_t t[TU];
    split_terms<TU>(v[e], t);
#pragma unroll
    for (int p = 0; p < TU; ++p) o[p][e] = t[p];
  }
#pragma unroll
  for (int p = 0; p < TU; ++p) *reinterpret_cast<u16x8 *>(stage + p * kTermElems + lane * kPitch + 8 * q) = o[p];
}

template <typename ST, int TU, int PRE>
__device__ __forceinline__ void stage_tile(uint16_t *stage, int w, int lane, const ST *X, const ST *Y, const float *Gn,
                                           const float *Go, int n, int ksteps, int64_t tile, int64_t ld,
                                           uint32_t valid, float alpha) {
  // two groups of 8 rows per trip: 16 to 48 loads in flight per lane
  for (int q = w; q < 2 * ksteps; q += 2 * kWaves) {
    stage_rows<ST, TU, PRE>(stage, q, lane, X, Y, Gn, Go, n, tile, ld, valid, alpha);
    if (q + kWaves < 2 * ksteps) stage_rows<ST, TU, PRE>(stage, q + kWaves, lane, X, Y, Gn, Go, n, tile, ld, valid, alpha);
  }
}

// acc[mt][nt] += P(rows 64w + 32mt ..) * staged tile (columns 32nt ..), all products (tp, tu) with tp + tu < max(TP, TU).
template <int TP, int TU>
__device__ __forceinline__ void product(f32x16 (&acc)[2][2], const uint16_t *stage, const u16x8 *__restrict__ frag,
                                        int w, int lane, int ksteps) {
  const int m = lane & 31, g = lane >> 5;
  constexpr int kMaxOrder = (TP > TU ? TP : TU) - 1;
  auto a_at = [&](int p, int mt, int kk) { return frag[((p * kMTiles + 2 * w + mt) * kKSteps + kk) * 64 + lane]; };
  u16x8 a[2][TP], an[2][TP];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int p = 0; p < TP; ++p) a[mt][p] = a_at(p, mt, 0);
  for (int kk = 0; kk < ksteps; ++kk) {
    const int kn = kk + 1 < ksteps ? kk + 1 : kk;  // next step's rows of P, under way while this step multiplies
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int p = 0; p < TP; ++p) an[mt][p] = a_at(p, mt, kn);
    u16x8 b[2][TU];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int p = 0; p < TU; ++p)
        b[nt][p] = *reinterpret_cast<const u16x8 *>(stage + p * kTermElems + (32 * nt + m) * kPitch + 16 * kk + 8 * g);
#pragma unroll
    for (int order = kMaxOrder; order >= 0; --order)  // smallest products first
#pragma unroll
      for (int tp = 0; tp < TP; ++tp) {
        const int tu = order - tp;
        if (tu < 0 || tu >= TU) continue;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int nt = 0; nt < 2; ++nt)
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[mt][tp]),
                                                                  __builtin_bit_cast(bf16x8, b[nt][tu]), acc[mt][nt], 0,
                                                                  0, 0);
      }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int p = 0; p < TP; ++p) a[mt][p] = an[mt][p];
  }
}

__device__ __forceinline__ void clear(f32x16 (&acc)[2][2]) {
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.f;
}

// mode 0: X <- P X.  mode 1 (ATC): X <- P (X - alpha*Y), Y <- P (Y + Gn - Go).
// mode 2 (ALG2): X <- P X - alpha * P Y, Y <- P Y + Gn - Go.
template <typename ST, int TP, int TU, int MODE>
__global__ __launch_bounds__(kThreads) void dense_phase_kernel(ST *X, ST *Y, const float *__restrict__ Gn,
                                                               const float *__restrict__ Go, int n, int64_t d,
                                                               int64_t ld, const u16x8 *__restrict__ frag, float alpha) {
  extern __shared__ uint16_t stage[];  // TU terms of the 64-column tile, [term][column][row]
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int m = lane & 31, g = lane >> 5;
  const int64_t tile = int64_t(blockIdx.x) * kCols;
  const uint32_t valid = uint32_t(d - tile < kCols ? d - tile : kCols);
  const int ksteps = (n + 15) / 16;
  const bool rows_mine = 64 * w < n;  // wavefront-uniform: this wavefront has output rows
  f32x16 acc[2][2];
  // element (mt, nt, r) of the accumulators: row 64w + 32mt + d_row(r, g), column tile + 32nt + m
  auto for_outputs = [&](auto &&fn) {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = 64 * w + 32 * mt + d_row(r, g), col = 32 * nt + m;
          if (row < n && uint32_t(col) < valid) fn(mt, nt, r, int64_t(row) * ld + tile + col);
        }
  };
  if constexpr (MODE == 0) {
    stage_tile<ST, TU, kPreX>(stage, w, lane, X, Y, Gn, Go, n, ksteps, tile, ld, valid, alpha);
    __syncthreads();
    if (rows_mine) {
      clear(acc);
      product<TP, TU>(acc, stage, frag, w, lane, ksteps);
      for_outputs([&](int mt, int nt, int r, int64_t at) { X[at] = from_f32<ST>(acc[mt][nt][r]); });
    }
  } else if constexpr (MODE == 1) {
    stage_tile<ST, TU, kPreXminusAlphaY>(stage, w, lane, X, Y, Gn, Go, n, ksteps, tile, ld, valid, alpha);
    __syncthreads();
    if (rows_mine) {
      clear(acc);
      product<TP, TU>(acc, stage, frag, w, lane, ksteps);
    }
    __syncthreads();  // every wavefront is done with the staged X tile (and has read all of X and Y it needs)
    if (rows_mine) for_outputs([&](int mt, int nt, int r, int64_t at) { X[at] = from_f32<ST>(acc[mt][nt][r]); });
    stage_tile<ST, TU, kPreTrack>(stage, w, lane, X, Y, Gn, Go, n, ksteps, tile, ld, valid, alpha);
    __syncthreads();
    if (rows_mine) {
      clear(acc);
      product<TP, TU>(acc, stage, frag, w, lane, ksteps);
      for_outputs([&](int mt, int nt, int r, int64_t at) { Y[at] = from_f32<ST>(acc[mt][nt][r]); });
    }
  } else {
    f32x16 py[2][2];
    stage_tile<ST, TU, kPreY>(stage, w, lane, X, Y, Gn, Go, n, ksteps, tile, ld, valid, alpha);
    __syncthreads();
    if (rows_mine) {
      clear(py);
      product<TP, TU>(py, stage, frag, w, lane, ksteps);
    }
    __syncthreads();
    stage_tile<ST, TU, kPreX>(stage, w, lane, X, Y, Gn, Go, n, ksteps, tile, ld, valid, alpha);
    __syncthreads();
    if (rows_mine) {
      clear(acc);
      product<TP, TU>(acc, stage, frag, w, lane, ksteps);
      for_outputs([&](int mt, int nt, int r, int64_t at) {
        X[at] = from_f32<ST>(fmaf(-alpha, py[mt][nt][r], acc[mt][nt][r]));
        Y[at] = from_f32<ST>(py[mt][nt][r] + Gn[at] - Go[at]);
      });
    }
  }
}

uint16_t bf16_rne_host(double v) {
  const float f = float(v);
  uint32_t u;
  __builtin_memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}
double bf16_value_host(uint16_t b) {
  const uint32_t u = uint32_t(b) << 16;
  float f;
  __builtin_memcpy(&f, &u, 4);
  return double(f);
}

template <typename ST, int TP, int TU>
int launch_mode(const Shape &s, int mode, void *X, void *Y, const float *Gn, const float *Go, float alpha,
                const uint16_t *frag, hipStream_t st) {
  const dim3 grid(ceil_div_i64(s.d, kCols));
  const size_t lds = size_t(TU) * kTermElems * sizeof(uint16_t);
  auto go = [&](auto *kernel) -> int {
    if (lds > 65536) {
      const hipError_t e =
          hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
      if (e != hipSuccess) return hip_rc(e);
    }
    kernel<<<grid, kThreads, lds, st>>>(static_cast<ST *>(X), static_cast<ST *>(Y), Gn, Go, s.n, s.d, s.ld,
                                        reinterpret_cast<const u16x8 *>(frag), alpha);
    return hip_rc(hipGetLastError());
  };
  switch (mode) {
    case 0: return go(&dense_phase_kernel<ST, TP, TU, 0>);
    case 1: return go(&dense_phase_kernel<ST, TP, TU, 1>);
    default: return go(&dense_phase_kernel<ST, TP, TU, 2>);
  }
}

}  // namespace

int dense_poly_terms(bool bf16_state) { return bf16_state ? 2 : 3; }
size_t dense_poly_words(int terms) { return size_t(terms) * kMTiles * kKSteps * 64 * 8; }

// P = p_K(W^T) in fp64 (n x n, row-major): p_0 = p_{-1} = I, p_{k+1} = (1+eta) W^T p_k - eta p_{k-1}.
void gossip_polynomial(const HostW &W, int K, double eta, std::vector<double> &P) {
  const int n = W.n;
  std::vector<double> prev(size_t(n) * n, 0.0), next(size_t(n) * n);
  P.assign(size_t(n) * n, 0.0);
  for (int i = 0; i < n; ++i) prev[size_t(i) * n + i] = P[size_t(i) * n + i] = 1.0;
  for (int k = 0; k < K; ++k) {
    for (int i = 0; i < n; ++i) {
      double *out = &next[size_t(i) * n];
      for (int c = 0; c < n; ++c) out[c] = 0.0;
      for (int t = W.rowptr[i]; t < W.rowptr[i + 1]; ++t) {  // row i lists (j, W_ji): the terms of worker i's sum
        const double wji = W.vals[t];
        const double *src = &P[size_t(W.colidx[t]) * n];
        for (int c = 0; c < n; ++c) out[c] += wji * src[c];
      }
      const double *pv = &prev[size_t(i) * n];
      for (int c = 0; c < n; ++c) out[c] = (1.0 + eta) * out[c] - eta * pv[c];
    }
    prev.swap(P);
    P.swap(next);
  }
}

// The bf16 terms of P in MFMA A-fragment order:
// frag[((term * 8 + mt) * 16 + kk) * 64 + lane][e] = term of P[32 mt + lane % 32][16 kk + 8 (lane / 32) + e], 0 past n.
bool build_dense_poly(const HostW &W, int K, double eta, int terms, std::vector<uint16_t> &frag) {
  const int n = W.n;
  if (n > kRowsMax || K < 0) return false;
  std::vector<double> P;
  gossip_polynomial(W, K, eta, P);
  frag.assign(dense_poly_words(terms), 0);
  for (int mt = 0; mt < kMTiles; ++mt)
    for (int kk = 0; kk < kKSteps; ++kk)
      for (int lane = 0; lane < 64; ++lane)
        for (int e = 0; e < 8; ++e) {
          const int i = 32 * mt + lane % 32, j = 16 * kk + 8 * (lane / 32) + e;
          if (i >= n || j >= n) continue;
          double rest = P[size_t(i) * n + j];
          for (int p = 0; p < terms; ++p) {
            const uint16_t b = bf16_rne_host(rest);
            frag[(((size_t(p) * kMTiles + mt) * kKSteps + kk) * 64 + lane) * 8 + e] = b;
            rest -= bf16_value_host(b);
          }
        }
  return true;
}

int launch_dense_phase(const Shape &s, int mode, void *X, void *Y, const float *Gn, const float *Go, float alpha,
                       const uint16_t *frag, void *stream) {
  auto st = static_cast<hipStream_t>(stream);
  return s.bf16 ? launch_mode<bf16_t, 2, 2>(s, mode, X, Y, Gn, Go, alpha, frag, st)
                : launch_mode<float, 3, 3>(s, mode, X, Y, Gn, Go, alpha, frag, st);
}

}  // namespace detag
