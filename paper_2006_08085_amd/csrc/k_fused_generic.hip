// K-round fused DeTAG phase for an arbitrary sparse gossip matrix with up to
// 256 workers and at most 8 neighbours per worker (e.g. a random regular graph
// with Metropolis weights).
//
// A block of 16 wavefronts owns 64 columns and all n rows of them.  Wavefront w
// owns the rows w, w+16, w+32, ... (RPT of them, RPT = 1, 2, 4, 8 or 16 by the
// number of workers); lane l owns column l.  Each lane
// keeps z_r and the velocity z_r - z_{r-1} of its own rows in registers; z_r
// of ALL rows also sits in LDS (16*RPT x 64 fp32), where the neighbours of a row
// are read.  Row indices are wavefront-uniform:
// the neighbour list of a row is a handful of scalars (16-bit LDS offsets packed
// in pairs, the weights), read once per kernel, and every LDS access is 64
// consecutive words, free of bank conflicts.  One round = read the neighbours
// from LDS, barrier, write the new values back, barrier.  HBM sees the state
// once per phase (16 B per element with bf16 state, 24 B with fp32); the rounds
// run at the LDS bandwidth, (deg+1) LDS words per
// output per round.  The kernel is kept within 64 VGPRs so that two blocks
// share a compute unit (2 x 64 KiB of LDS): one block's loads and stores then
// run under the other's rounds.
//
// Paper: Algorithm 3 (accelerated gossip) and Algorithm 2 / the matrix form in
// the proof of Theorem 3 (phase update).
#include "detag_internal.h"
#include "dev_common.hpp"
#include "noise_dev.hpp"

namespace detag {
namespace {

constexpr int kWaves = 16, kThreads = 64 * kWaves, kCols = 64, RPTMax = 16, kRowsMax = kWaves * RPTMax;  // 256 rows

// Rows per wavefront (RPT below): the smallest of 1, 2, 4, 8, 16 that gives all n workers a slot (16 * RPT >= n).
// A block's arithmetic, LDS footprint and table are proportional to its slots, not to n, so a small graph on
// the 256-slot layout would pay for 256 workers (measured on a 7-worker ring: 18 times the time per byte of the
// 256-worker case).
int rows_per_wave(int n) {
  int r = 1;
  while (r < RPTMax && kWaves * r < n) r *= 2;
  return r;
}

// Table words per row: DEG/2 words of packed 16-bit LDS byte offsets, then the
// neighbour weights (one word if they are all equal, else DEG).  W_ii is not
// stored: a round is evaluated in velocity form, v = z_r - z_{r-1},
//   v_i <- (1+eta) * sum_j W_ji (z_j - z_i) + eta * v_i,   z_i <- z_i + v_i,
// in which equal values across the workers are a fixed point exactly whatever
// the rounding of the weights (the worker mean does not drift with K) and the
// only rounding at the magnitude of z is the last add.
// Padding entries point at the row itself (difference zero).
constexpr int table_stride(int deg, bool uniform) { return deg / 2 + (uniform ? 1 : deg); }

template <int DEG, bool UNI>
struct RowTab {
  uint32_t w[table_stride(DEG, UNI)];
  __device__ __forceinline__ uint32_t off(int k) const { return (k & 1) ? w[k >> 1] >> 16 : w[k >> 1] & 0xffffu; }
  __device__ __forceinline__ float val(int k) const { return __uint_as_float(w[DEG / 2 + (UNI ? 0 : k)]); }
};

// One round for this lane's rows, with the velocity kept divided by (1+eta) (and, for rows whose neighbour
// weights are all equal, also by that weight; the table then holds (1+eta)*weight, see scale_uniform_weights):
//   u <- sum_k W_ji (lds[j] - z) + eta * u;   z <- z + (1+eta) * u;   then publish z.
// Two multiplications fewer per output and round than with the velocity itself; the kernel issues about as many
// vector-ALU cycles as LDS cycles per round, so they count.
template <int DEG, bool UNI, bool FIRST, int RPT>
__device__ __forceinline__ void round_step(float (&z)[RPT], float (&u)[RPT], const char *lds_b, float *lds, int w,
                                           int lane, RowTab<DEG, UNI> (&tab)[RPT], float cm, float eta) {
  // The packed offset words are made opaque once per round: otherwise their 16-bit halves are unpacked ahead
  // of the round loop into 4*DEG*... scalar registers of their own, which do not fit beside the table at two
  // blocks per compute unit and end up spilled.
#pragma unroll
  for (int r = 0; r < RPT; ++r)
#pragma unroll
    for (int q = 0; q < DEG / 2; ++q) asm volatile("" : "+s"(tab[r].w[q]));
  const uint32_t lane4 = uint32_t(lane) * 4u;
  auto nb = [&](int r, int k) { return *reinterpret_cast<const float *>(lds_b + (tab[r].off(k) + lane4)); };
#pragma unroll
  for (int r = 0; r < RPT; ++r) {
    float acc;
    if constexpr (UNI) {
      // pairwise tree: DEG equal values sum exactly, so s - DEG*z is exactly zero for them
      float s[DEG];
#pragma unroll
      for (int k = 0; k < DEG; ++k) s[k] = nb(r, k);
#pragma unroll
      for (int len = DEG / 2; len >= 1; len /= 2)
#pragma unroll
        for (int k = 0; k < len; ++k) s[k] += s[k + len];
      acc = fmaf(-float(DEG), z[r], s[0]);
    } else {
      acc = 0.f;
#pragma unroll
      for (int k = 0; k < DEG; ++k) acc = fmaf(tab[r].val(k), nb(r, k) - z[r], acc);
    }
    u[r] = FIRST ? acc : fmaf(eta, u[r], acc);
  }
  __syncthreads();  // every read of z_r is done
#pragma unroll
  for (int r = 0; r < RPT; ++r) {
    z[r] = fmaf(UNI ? tab[r].val(0) : cm, u[r], z[r]);
    lds[(w + kWaves * r) * kCols + lane] = z[r];
  }
  __syncthreads();  // z_{r+1} is visible
}

// For rows with one weight, the table's weight word becomes (1+eta)*weight, a wavefront-uniform value kept in a
// scalar register like the weight it replaces.
template <int DEG, bool UNI, int RPT>
__device__ __forceinline__ void scale_uniform_weights(RowTab<DEG, UNI> (&tab)[RPT], float cm) {
  if constexpr (UNI) {
#pragma unroll
    for (int r = 0; r < RPT; ++r)
      tab[r].w[DEG / 2] = __builtin_amdgcn_readfirstlane(__float_as_uint(cm * tab[r].val(0)));
  }
}

// K >= 1 rounds from z_{-1} = z_0 = z.  Result in z; v is scratch.  The table's weights are already scaled.
template <int DEG, bool UNI, int RPT>
__device__ __forceinline__ void gossip(float (&z)[RPT], float (&v)[RPT], float *lds, int w, int lane,
                                       RowTab<DEG, UNI> (&tab)[RPT], float eta, int K) {
  const float cm = 1.f + eta;
  const char *lds_b = reinterpret_cast<const char *>(lds);
#pragma unroll
  for (int r = 0; r < RPT; ++r) lds[(w + kWaves * r) * kCols + lane] = z[r];
  __syncthreads();
  round_step<DEG, UNI, true, RPT>(z, v, lds_b, lds, w, lane, tab, cm, eta);
  for (int r = 1; r < K; ++r) round_step<DEG, UNI, false, RPT>(z, v, lds_b, lds, w, lane, tab, cm, eta);
}

// Window of row i of the tile; rows >= n get an empty window (loads give 0, stores are dropped).
template <typename E>
__device__ __forceinline__ rsrc_t win(const E *base, int64_t tile, int64_t ld, int i, int n, uint32_t valid) {
  return row_of(base, tile, ld, i < n ? i : 0, i < n ? valid : 0u);
}

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


// Gradient query of the diagonal-quadratic objective and the ATC phase in one pass (the form
// detag_step_quadratic takes on a context of this kernel family):
//   G+ = h*(X - b) + sigma*z;  X+ = M(X - alpha*Y);  Y+ = M(Y + G+ - G),
// G updated in place (row by row, the old value read just before the new one is stored).  Same three arrays
// per lane as the plain ATC phase: the gradient is consumed and stored inside the load loop.  Per element it
// reads X, Y (state type), G, b (fp32) and writes X, Y, G, where the gradient kernel followed by the phase moves
// X twice more and the gradient three times.  The counter-based noise shares one Philox block among the four
// lanes of a quad when a wavefront has at least four rows (see quad_transpose); with fewer rows per wavefront
// every lane evaluates the block of its own row and keeps one of the four normals.
template <typename ST, int DEG, bool UNI, int RPT, bool HPW>
__global__ __launch_bounds__(kThreads, 8) void fused_generic_quadratic_kernel(
    ST *X, ST *Y, float *G, const float *__restrict__ h, const float *__restrict__ b, int n, int64_t d, int64_t ld,
    const uint32_t *__restrict__ table, float eta, float alpha, int K, float sigma, uint32_t seed_lo, uint32_t seed_hi,
    uint32_t step) {
  extern __shared__ float lds[];  // 16*RPT x 64
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int64_t tile = int64_t(blockIdx.x) * kCols;
  const uint32_t valid = uint32_t(d - tile < kCols ? d - tile : kCols);
  const uint32_t so = lane * uint32_t(sizeof(ST)), fo = lane * 4u;
  const unsigned j = lane & 3u;
  const uint64_t q = uint64_t(tile + lane) >> 2;  // Philox block = 4 columns; tiles start at multiples of 64
  constexpr int TS = table_stride(DEG, UNI);
  RowTab<DEG, UNI> tab[RPT];
#pragma unroll
  for (int r = 0; r < RPT; ++r)
#pragma unroll
    for (int t = 0; t < TS; ++t) tab[r].w[t] = table[(w * RPT + r) * TS + t];
  scale_uniform_weights<DEG, UNI, RPT>(tab, 1.f + eta);
  const float hc = HPW ? 0.f : buf_load<float>(make_rsrc(h + tile, valid * 4u), fo);
  float cur[RPT], prev[RPT], v0[RPT];
  auto row = [&](int r) { return w + kWaves * r; };
  constexpr int kBatch = RPT < 4 ? RPT : 4;
#pragma unroll
  for (int r0 = 0; r0 < RPT; r0 += kBatch) {
    // the batch's noise first, its loads after: generated under the loads, the Philox state and the sixteen
    // values in flight are live together and the kernel no longer fits two blocks per compute unit without spills
    float z[4] = {0.f, 0.f, 0.f, 0.f};
    if (sigma != 0.f) {
      if constexpr (kBatch == 4) {  // lane j of a quad: the block of row r0 + j, then a 4x4 transpose
        normal4(q, uint32_t(w + kWaves * (r0 + int(j))), step, seed_lo, seed_hi, z);
        quad_transpose(z, j);
      } else {
#pragma unroll
        for (int t = 0; t < kBatch; ++t) {
          float zz[4];
          normal4(q, uint32_t(row(r0 + t)), step, seed_lo, seed_hi, zz);
          z[t] = j == 0 ? zz[0] : j == 1 ? zz[1] : j == 2 ? zz[2] : zz[3];
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    float x[kBatch], y[kBatch], go[kBatch], bb[kBatch], hh[HPW ? kBatch : 1];
#pragma unroll
    for (int t = 0; t < kBatch; ++t) {
      x[t] = buf_load<ST>(win(X, tile, ld, row(r0 + t), n, valid), so);
      y[t] = buf_load<ST>(win(Y, tile, ld, row(r0 + t), n, valid), so);
      go[t] = buf_load<float>(win(G, tile, ld, row(r0 + t), n, valid), fo);
      bb[t] = buf_load<float>(win(b, tile, ld, row(r0 + t), n, valid), fo);
      if constexpr (HPW) hh[t] = buf_load<float>(win(h, tile, ld, row(r0 + t), n, valid), fo);
    }
#pragma unroll
    for (int t = 0; t < kBatch; ++t) {
      const float g = fmaf(sigma, z[t], (HPW ? hh[t] : hc) * (x[t] - bb[t]));
      cur[r0 + t] = fmaf(-alpha, y[t], x[t]);
      v0[r0 + t] = y[t] + g - go[t];
      pin_vgpr(v0[r0 + t]);
      buf_store<float>(win(G, tile, ld, row(r0 + t), n, valid), fo, g);
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

template <typename ST, int DEG, bool UNI>
int launch_q(const Shape &s, const uint32_t *table, void *X, void *Y, float *G, const float *h, bool hpw, const float *b,
             float alpha, int K, float eta, float sigma, uint64_t seed, uint32_t step, void *stream) {
  const dim3 grid(ceil_div_i64(s.d, kCols));
  auto st = static_cast<hipStream_t>(stream);
  ST *x = static_cast<ST *>(X), *y = static_cast<ST *>(Y);
  const uint32_t slo = uint32_t(seed & 0xffffffffu), shi = uint32_t(seed >> 32);
#define DETAG_QUAD(R, HPW)                                                                                          \
  fused_generic_quadratic_kernel<ST, DEG, UNI, R, HPW>                                                              \
      <<<grid, kThreads, size_t(kWaves) * R * kCols * sizeof(float), st>>>(x, y, G, h, b, s.n, s.d, s.ld, table, eta, \
                                                                           alpha, K, sigma, slo, shi, step)
#define DETAG_RPT(R)                                            \
  case R:                                                       \
    if (hpw) DETAG_QUAD(R, true); else DETAG_QUAD(R, false);    \
    break
  switch (rows_per_wave(s.n)) {
    DETAG_RPT(1);
    DETAG_RPT(2);
    DETAG_RPT(4);
    DETAG_RPT(8);
    DETAG_RPT(16);
    default: return -1;
  }
#undef DETAG_RPT
#undef DETAG_QUAD
  return hip_rc(hipGetLastError());
}

template <typename ST>
int launch_qt(const Shape &s, const uint32_t *table, int deg, bool uni, void *X, void *Y, float *G, const float *h,
              bool hpw, const float *b, float alpha, int K, float eta, float sigma, uint64_t seed, uint32_t step,
              void *stream) {
#define DETAG_CASE(DG)                                                                                          \
  case DG:                                                                                                      \
    return uni ? launch_q<ST, DG, true>(s, table, X, Y, G, h, hpw, b, alpha, K, eta, sigma, seed, step, stream)  \
               : launch_q<ST, DG, false>(s, table, X, Y, G, h, hpw, b, alpha, K, eta, sigma, seed, step, stream)
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

int launch_fused_generic_quadratic(const Shape &s, const DevCsr &w, void *X, void *Y, float *G, const float *h,
                                   bool h_per_worker, const float *b, float alpha, int K, float eta, float sigma,
                                   uint64_t seed, uint32_t step, void *stream) {
  if (K < 1 || !w.ell_table) return -1;
  return s.bf16 ? launch_qt<bf16_t>(s, w.ell_table, w.ell_deg, w.ell_uniform, X, Y, G, h, h_per_worker, b, alpha, K, eta,
                                    sigma, seed, step, stream)
                : launch_qt<float>(s, w.ell_table, w.ell_deg, w.ell_uniform, X, Y, G, h, h_per_worker, b, alpha, K, eta,
                                   sigma, seed, step, stream);
}

}  // namespace detag
