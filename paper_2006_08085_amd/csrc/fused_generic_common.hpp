// Shared by the LDS-resident kernels: K-round fused DeTAG phase for an arbitrary sparse gossip matrix with up to
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
#pragma once

#include "detag_internal.h"
#include "dev_common.hpp"

namespace detag {
namespace lds_tile {

constexpr int kWaves = 16, kThreads = 64 * kWaves, kCols = 64, kRptMax = 16, kRowsMax = kWaves * kRptMax;  // 256 rows

// Rows per wavefront (RPT below): the smallest of 1, 2, 4, 8, 16 that gives all n workers a slot (16 * RPT >= n).
// A block's arithmetic, LDS footprint and table are proportional to its slots, not to n, so a small graph on
// the 256-slot layout would pay for 256 workers (measured on a 7-worker ring: 18 times the time per byte of the
// 256-worker case).
inline int rows_per_wave(int n) {
  int r = 1;
  while (r < kRptMax && kWaves * r < n) r *= 2;
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

}  // namespace lds_tile
}  // namespace detag
