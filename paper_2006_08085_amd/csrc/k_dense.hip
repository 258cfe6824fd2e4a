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
// for bf16 state 2 + 2 terms and 3 products (a bf16 input is its own first
// term).  An infinite input leaves NaN in its column (Inf - Inf in the split),
// where the round-by-round kernels leave Inf or NaN.
//
// One block = 64 columns, 4 wavefronts, three blocks to a compute unit (two with fp32 state, whose three-term
// operands need the registers).  The input of a pass is staged in units of
// 128 workers.  Staging: lane = column, a wavefront loads groups of 8 consecutive rows (coalesced row segments),
// applies the phase's elementwise part (X - alpha Y, Y + Gnew - Gold), splits, and writes one 16-byte word per
// term to LDS laid out [term][column][row] -- exactly the B operand (column m, k = 8g..8g+7) of the MFMA.
// Product: wavefront w owns output rows 64w..64w+63 (two 32-row tiles) of both 32-column tiles; the A operand
// comes from a copy of P the host pre-arranged in fragment order (one 1 KiB coalesced load per tile and k-step,
// served by L2, requested a few k-steps ahead).  The result leaves through LDS as well: a wavefront transposes its
// accumulators 16 rows at a time in a scratch area of its own, so that it stores whole row segments with lane =
// column like every other kernel here (storing the accumulator layout directly, 32 columns of two rows per
// instruction, ran at a third of the rate).  MFMA operand layout (lane l, m = l % 32, g = l / 32):
// A: row m, k = 8g..8g+7;  B: column m, k = 8g..8g+7;  D: column m, register r -> row 8*(r/4) + 4g + r%4.
#include "detag_internal.h"
#include "dev_common.hpp"

namespace detag {
namespace {

constexpr int kCols = 64, kThreads = 256, kWaves = 4;
constexpr int kRowsMax = 256, kMTiles = kRowsMax / 32, kKSteps = kRowsMax / 16;
constexpr int kUnitSteps = 8;    // k-steps (of 16 rows) staged in LDS at a time
constexpr int kOutPitch = 72;    // floats per row of a wavefront's 16 x 64 output scratch: rows 4 apart are 32 banks apart
constexpr int kOutBytes = kWaves * 16 * kOutPitch * 4;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ int d_row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

// The bf16 terms of 8 consecutive rows of one column, one 16-byte word per term (row e in 16-bit element e).
// Three terms (fp32 state) are cut by truncation: t0 = the upper 16 bits of v, t1 = the upper 16 bits of v - t0, ...
// hold all 24 significant bits, for a mask and a subtraction per term.  Two terms (bf16 state, whose stored values
// are their own first term; only the phase's elementwise part makes a second one) are rounded to nearest, which
// leaves 2^-17 of the value instead of 2^-16 behind.
template <int TU>
__device__ __forceinline__ void split_rows(const float (&v)[8], uint4 (&o)[TU]) {
  if constexpr (TU == 3) {
    float r[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = v[e];
#pragma unroll
    for (int p = 0; p < TU; ++p) {
      // the upper halves of two neighbouring rows share a 32-bit word, the even row in the lower half
      auto pair = [&](int e) {
        return __builtin_amdgcn_perm(__float_as_uint(r[e + 1]), __float_as_uint(r[e]), 0x07060302u);
      };
      o[p].x = pair(0), o[p].y = pair(2), o[p].z = pair(4), o[p].w = pair(6);
      if (p + 1 < TU) {
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] -= __uint_as_float(__float_as_uint(r[e]) & 0xffff0000u);
      }
    }
  } else {
    uint32_t t[TU][8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float r = v[e];
#pragma unroll
      for (int p = 0; p < TU; ++p) {
        t[p][e] = bf16_bits_rne(r);
        r -= __uint_as_float(t[p][e] << 16);
      }
    }
#pragma unroll
    for (int p = 0; p < TU; ++p) {
      o[p].x = t[p][0] | (t[p][1] << 16), o[p].y = t[p][2] | (t[p][3] << 16);
      o[p].z = t[p][4] | (t[p][5] << 16), o[p].w = t[p][6] | (t[p][7] << 16);
    }
  }
}

// What is multiplied by P in a pass.
enum Pre : int { kPreX = 0, kPreXminusAlphaY = 1, kPreTrack = 2, kPreY = 3 };

// Geometry of a kernel compiled for KS k-steps (n <= 16 KS): the staged unit holds KU k-steps, one column of one term
// takes kPitch bf16 (8 more than its rows, so that 16 consecutive columns start in 16 different groups of 4 banks).
template <int KS>
struct Geo {
  static constexpr int KU = KS < kUnitSteps ? KS : kUnitSteps;
  static constexpr int kUnits = KS / KU;
  static constexpr int kPitch = 16 * KU + 8;
  static constexpr int kTermElems = kCols * kPitch;
  static constexpr int kGroups = 2 * KU / kWaves;  // groups of 8 rows a wavefront stages per unit (KS >= 2)
};

// One unit (rows 16 KU u ...) of the block's 64 columns -> the elementwise part -> TU bf16 terms in LDS, laid out
// [term][column][row].  Lane = column; wavefront w takes the groups of 8 rows w, w+4, ...; rows >= n are staged as
// zeros (their resource has no valid bytes).
template <typename ST, int TU, int PRE, int KS>
__device__ __forceinline__ void stage_unit(uint16_t *stage, int u, int w, int lane, const ST *X, const ST *Y,
                                           const float *Gn, const float *Go, int n, int64_t tile, int64_t ld,
                                           uint32_t valid, float alpha) {
  using G = Geo<KS>;
  const uint32_t so = lane * uint32_t(sizeof(ST)), fo = lane * 4u;
  // groups whose loads are in flight together: 32 rows of one array, 16 rows of two or three (the accumulators
  // of earlier units are live meanwhile)
  constexpr int kChunk = PRE != kPreX && PRE != kPreY && G::kGroups > 2 ? 2 : G::kGroups;
#pragma unroll
  for (int c0 = 0; c0 < G::kGroups; c0 += kChunk) {
    float v[kChunk][8];
#pragma unroll
    for (int c = 0; c < kChunk; ++c) {
      const int row0 = 16 * G::KU * u + 8 * (w + kWaves * (c0 + c));  // wavefront-uniform
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        // a row >= n gets a resource without valid bytes
        const uint32_t ok = row0 + e < n ? valid : 0u;
        const int rr = row0 + e < n ? row0 + e : 0;
        if constexpr (PRE == kPreX) {
          v[c][e] = buf_load<ST>(row_of(X, tile, ld, rr, ok), so);
        } else if constexpr (PRE == kPreY) {
          v[c][e] = buf_load<ST>(row_of(Y, tile, ld, rr, ok), so);
        } else if constexpr (PRE == kPreXminusAlphaY) {
          const float x = buf_load<ST>(row_of(X, tile, ld, rr, ok), so), y = buf_load<ST>(row_of(Y, tile, ld, rr, ok), so);
          v[c][e] = fmaf(-alpha, y, x);
        } else {
          const float y = buf_load<ST>(row_of(Y, tile, ld, rr, ok), so);
          const float gn = buf_load<float>(row_of(Gn, tile, ld, rr, ok), fo);
          const float go = buf_load<float>(row_of(Go, tile, ld, rr, ok), fo);
          v[c][e] = y + gn - go;
        }
      }
    }
    // every load of the chunk is issued before the first value is used: left alone, the compiler waits for the
    // first rows after a handful of loads to save registers, and the memory pipeline runs dry
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int c = 0; c < kChunk; ++c) {
      uint4 o[TU];
      split_rows<TU>(v[c], o);
#pragma unroll
      for (int p = 0; p < TU; ++p)
        *reinterpret_cast<uint4 *>(stage + p * G::kTermElems + lane * G::kPitch + 8 * (w + kWaves * (c0 + c))) = o[p];
    }
    if (c0 + kChunk < G::kGroups) __builtin_amdgcn_sched_barrier(0);  // keep the chunks' loads apart
  }
}

// The rows of P a wavefront multiplies by: its two 32-row tiles, TP terms, k-step kk.
template <int TP>
struct AFrag {
  u16x8 t[2][TP];
};
template <int TP>
__device__ __forceinline__ AFrag<TP> load_a(const u16x8 *__restrict__ frag, int w, int lane, int kk) {
  AFrag<TP> a;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int p = 0; p < TP; ++p) a.t[mt][p] = frag[((p * kMTiles + 2 * w + mt) * kKSteps + kk) * 64 + lane];
  return a;
}

// acc[mt][nt] += P(rows 64w + 32mt .., k-steps of unit u) * staged unit (columns 32nt ..): all products (tp, tu) with
// tp + tu < max(TP, TU), the smallest first.  `ring` holds the unit's first DEPTH k-steps' rows of P on entry (loaded
// before the barrier that publishes the unit); the rows DEPTH steps ahead are requested as soon as a step is used.
template <int TP, int TU, int KS, int DEPTH>
__device__ __forceinline__ void product_unit(f32x16 (&acc)[2][2], const uint16_t *stage, AFrag<TP> (&ring)[DEPTH],
                                             const u16x8 *__restrict__ frag, int u, int w, int lane) {
  using G = Geo<KS>;
  const int m = lane & 31, g = lane >> 5;
  constexpr int kMaxOrder = (TP > TU ? TP : TU) - 1;
  // the fence at the end of a step keeps the compiler from pulling every later step's reads to the front (and their
  // registers with them); the other wavefronts of the SIMD cover a step's LDS latency
#pragma unroll
  for (int s = 0; s < G::KU; ++s) {
    u16x8 b[2][TU];
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int p = 0; p < TU; ++p)
        b[nt][p] = *reinterpret_cast<const u16x8 *>(stage + p * G::kTermElems + (32 * nt + m) * G::kPitch + 16 * s + 8 * g);
    const AFrag<TP> &a = ring[s % DEPTH];
#pragma unroll
    for (int order = kMaxOrder; order >= 0; --order)
#pragma unroll
      for (int tp = 0; tp < TP; ++tp) {
        const int tu = order - tp;
        if (tu < 0 || tu >= TU) continue;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int nt = 0; nt < 2; ++nt)
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a.t[mt][tp]),
                                                                  __builtin_bit_cast(bf16x8, b[nt][tu]), acc[mt][nt], 0,
                                                                  0, 0);
      }
    if (s + DEPTH < G::KU) ring[s % DEPTH] = load_a<TP>(frag, w, lane, G::KU * u + s + DEPTH);
    __builtin_amdgcn_sched_barrier(0);
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

// acc = P * (the pass's input), unit by unit.  `fresh` = nothing has used LDS yet.  Ends with a barrier: every
// wavefront is done with the staged input.
template <typename ST, int TP, int TU, int PRE, int KS>
__device__ __forceinline__ void pass(f32x16 (&acc)[2][2], uint16_t *stage, bool fresh, bool rows_mine, int w, int lane,
                                     const ST *X, const ST *Y, const float *Gn, const float *Go, int n, int64_t tile,
                                     int64_t ld, uint32_t valid, float alpha, const u16x8 *__restrict__ frag) {
  using G = Geo<KS>;
  constexpr int kDepth = 2;  // k-steps the rows of P are requested ahead (three cost registers, and spills, for nothing)
#pragma unroll
  for (int u = 0; u < G::kUnits; ++u) {
    if (u > 0 || !fresh) __syncthreads();  // every wavefront is done with what LDS held
    stage_unit<ST, TU, PRE, KS>(stage, u, w, lane, X, Y, Gn, Go, n, tile, ld, valid, alpha);
    __builtin_amdgcn_sched_barrier(0);  // the rows of P are requested after the staging loads, not among them
    AFrag<TP> ring[kDepth];
    if (rows_mine) {
#pragma unroll
      for (int s = 0; s < kDepth; ++s) ring[s] = load_a<TP>(frag, w, lane, G::KU * u + s);
    }
    __syncthreads();
    if (u == 0) clear(acc);
    if (rows_mine) product_unit<TP, TU, KS, kDepth>(acc, stage, ring, frag, u, w, lane);
  }
  __syncthreads();
}

// The wavefront's 64 x 64 results, 16 rows at a time through its scratch area: accumulator layout in, rows out.
// fn(row, value) stores row `row` of the block's columns, lane = column.
template <typename F>
__device__ __forceinline__ void write_out(const f32x16 (&acc)[2][2], float *scratch, int w, int lane, int n, F &&fn) {
  const int m = lane & 31, g = lane >> 5;
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int h = 0; h < 2; ++h) {  // registers 8h..8h+7 hold rows 16h..16h+15 of the 32-row tile
      const int row0 = 64 * w + 32 * mt + 16 * h;
      if (row0 >= n) continue;  // wavefront-uniform
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 8; ++r) scratch[d_row(r, g) * kOutPitch + 32 * nt + m] = acc[mt][nt][8 * h + r];
      float v[16];
#pragma unroll
      for (int q = 0; q < 16; ++q) v[q] = scratch[q * kOutPitch + lane];
#pragma unroll
      for (int q = 0; q < 16; ++q)
        if (row0 + q < n) fn(row0 + q, v[q]);
    }
}

// mode 0: X <- P X.  mode 1 (ATC): X <- P (X - alpha*Y), Y <- P (Y + Gn - Go).
// mode 2 (ALG2): X <- P X - alpha * P Y = P (X - alpha*Y) (P is linear), Y <- P Y + Gn - Go.  n <= 16 KS.
// A pass writes its result once every wavefront has staged all the pass reads of the array it overwrites.
template <typename ST, int TP, int TU, int MODE, int KS>
__global__ __launch_bounds__(kThreads, TP >= 3 ? 2 : 3) void dense_phase_kernel(ST *X, ST *Y, const float *__restrict__ Gn,
                                                                  const float *__restrict__ Go, int n, int64_t d,
                                                                  int64_t ld, const u16x8 *__restrict__ frag,
                                                                  float alpha) {
  extern __shared__ uint16_t stage[];  // TU terms of one unit of the 64-column tile; afterwards the output scratch
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int64_t tile = int64_t(blockIdx.x) * kCols;
  const uint32_t valid = uint32_t(d - tile < kCols ? d - tile : kCols);
  const bool rows_mine = 64 * w < n;  // wavefront-uniform: this wavefront has output rows
  const uint32_t so = lane * uint32_t(sizeof(ST)), fo = lane * 4u;
  float *scratch = reinterpret_cast<float *>(stage) + w * 16 * kOutPitch;
  f32x16 acc[2][2];
  auto store_rows = [&](ST *out) {
    if (rows_mine)
      write_out(acc, scratch, w, lane, n, [&](int row, float v) { buf_store<ST>(row_of(out, tile, ld, row, valid), so, v); });
  };
  if constexpr (MODE == 0) {
    pass<ST, TP, TU, kPreX, KS>(acc, stage, true, rows_mine, w, lane, X, Y, Gn, Go, n, tile, ld, valid, alpha, frag);
    store_rows(X);
  } else {
    pass<ST, TP, TU, kPreXminusAlphaY, KS>(acc, stage, true, rows_mine, w, lane, X, Y, Gn, Go, n, tile, ld, valid, alpha,
                                           frag);
    store_rows(X);
    if constexpr (MODE == 1) {
      pass<ST, TP, TU, kPreTrack, KS>(acc, stage, false, rows_mine, w, lane, X, Y, Gn, Go, n, tile, ld, valid, alpha, frag);
      store_rows(Y);
    } else {
      pass<ST, TP, TU, kPreY, KS>(acc, stage, false, rows_mine, w, lane, X, Y, Gn, Go, n, tile, ld, valid, alpha, frag);
      if (rows_mine)
        write_out(acc, scratch, w, lane, n, [&](int row, float v) {
          const float gn = buf_load<float>(row_of(Gn, tile, ld, row, valid), fo);
          const float go = buf_load<float>(row_of(Go, tile, ld, row, valid), fo);
          buf_store<ST>(row_of(Y, tile, ld, row, valid), so, v + gn - go);
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

template <typename ST, int TP, int TU, int KS>
int launch_ks(const Shape &s, int mode, void *X, void *Y, const float *Gn, const float *Go, float alpha,
              const uint16_t *frag, hipStream_t st) {
  const dim3 grid(ceil_div_i64(s.d, kCols));
  const size_t staged = size_t(TU) * Geo<KS>::kTermElems * sizeof(uint16_t);  // at most 3 * 64 * 136 * 2 bytes
  const size_t lds = staged > size_t(kOutBytes) ? staged : size_t(kOutBytes);
  auto go = [&](auto *kernel) -> int {
    kernel<<<grid, kThreads, lds, st>>>(static_cast<ST *>(X), static_cast<ST *>(Y), Gn, Go, s.n, s.d, s.ld,
                                        reinterpret_cast<const u16x8 *>(frag), alpha);
    return hip_rc(hipGetLastError());
  };
  switch (mode) {
    case 0: return go(&dense_phase_kernel<ST, TP, TU, 0, KS>);
    case 1: return go(&dense_phase_kernel<ST, TP, TU, 1, KS>);
    default: return go(&dense_phase_kernel<ST, TP, TU, 2, KS>);
  }
}

// The kernel is compiled for 2, 4, 8 and 16 k-steps of 16 workers: the smallest that covers n.
template <typename ST, int TP, int TU>
int launch_mode(const Shape &s, int mode, void *X, void *Y, const float *Gn, const float *Go, float alpha,
                const uint16_t *frag, hipStream_t st) {
  if (s.n <= 32) return launch_ks<ST, TP, TU, 2>(s, mode, X, Y, Gn, Go, alpha, frag, st);
  if (s.n <= 64) return launch_ks<ST, TP, TU, 4>(s, mode, X, Y, Gn, Go, alpha, frag, st);
  if (s.n <= 128) return launch_ks<ST, TP, TU, 8>(s, mode, X, Y, Gn, Go, alpha, frag, st);
  return launch_ks<ST, TP, TU, 16>(s, mode, X, Y, Gn, Go, alpha, frag, st);
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
