// Gradient query of the diagonal-quadratic objective fused into the ATC phase of the LDS-resident kernels
// (layout and round arithmetic in fused_generic_common.hpp).
//
// Paper: gradient query and phase update of Algorithm 2 (matrix form in the proof of Theorem 3), Algorithm 3.
#include "fused_generic_common.hpp"
#include "noise_dev.hpp"

namespace detag {
namespace {

using namespace lds_tile;

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

}  // namespace

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
