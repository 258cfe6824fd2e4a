// Streaming kernels: one gossip round over a CSR gossip matrix, the tracker
// update, the model update, D-PSGD.  Every kernel is a pure pass over n x d
// elements, d contiguous; threads own VEC adjacent columns and walk the rows,
// so each lane issues 16-byte (fp32) or 8-byte (bf16) accesses and a wavefront
// touches 1 KiB (or 512 B) of one row at a time.
//
// Paper: the gossip sum is the gossip equation of the "Protocol Layer"
// subsection; the momentum form is the loop body of Algorithm 3; the tracker
// and model updates are the end-of-phase lines of Algorithm 2.
#include "dev_common.hpp"
#include "detag_internal.h"

namespace detag {
namespace {

constexpr int kThreads = 256;

// Streamed data (touched once per kernel) goes through non-temporal accesses: on the 64 x 11.2 M fp32 matrices the
// update-and-track pass takes 2.78 ms with them against 3.14 ms without (0.77 against 0.68 of HBM peak), the
// tracker update 1.75 against 2.06 ms.  Rows that neighbours read again within a kernel (NT = false) stay cached.
typedef float vf4_t __attribute__((ext_vector_type(4)));
typedef uint32_t vu2_t __attribute__((ext_vector_type(2)));

template <bool NT>
__device__ __forceinline__ float load_one(const float *p) { return NT ? __builtin_nontemporal_load(p) : *p; }
template <bool NT>
__device__ __forceinline__ float load_one(const bf16_t *p) {
  return __uint_as_float(uint32_t(NT ? __builtin_nontemporal_load(&p->bits) : p->bits) << 16);
}
__device__ __forceinline__ void store_one(float *p, float v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void store_one(bf16_t *p, float v) { __builtin_nontemporal_store(bf16_bits_rne(v), &p->bits); }

template <typename ST, int VEC, bool NT = true>
__device__ __forceinline__ void load_vec(const ST *p, int valid, float (&v)[VEC]) {
  if constexpr (VEC == 4) {
    if (valid >= 4) {
      if constexpr (sizeof(ST) == 4) {
        const vf4_t *q = reinterpret_cast<const vf4_t *>(p);
        const vf4_t t = NT ? __builtin_nontemporal_load(q) : *q;
        v[0] = t.x, v[1] = t.y, v[2] = t.z, v[3] = t.w;
      } else {
        const vu2_t *q = reinterpret_cast<const vu2_t *>(p);
        const vu2_t t = NT ? __builtin_nontemporal_load(q) : *q;
        v[0] = __uint_as_float(t.x << 16), v[1] = __uint_as_float(t.x & 0xffff0000u);
        v[2] = __uint_as_float(t.y << 16), v[3] = __uint_as_float(t.y & 0xffff0000u);
      }
      return;
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) v[e] = e < valid ? load_one<NT>(p + e) : 0.f;
}

template <typename ST, int VEC>
__device__ __forceinline__ void store_vec(ST *p, int valid, const float (&v)[VEC]) {
  if constexpr (VEC == 4) {
    if (valid >= 4) {
      if constexpr (sizeof(ST) == 4) {
        const vf4_t t = {v[0], v[1], v[2], v[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<vf4_t *>(p));
      } else {
        vu2_t t;
        t.x = uint32_t(bf16_bits_rne(v[0])) | (uint32_t(bf16_bits_rne(v[1])) << 16);
        t.y = uint32_t(bf16_bits_rne(v[2])) | (uint32_t(bf16_bits_rne(v[3])) << 16);
        __builtin_nontemporal_store(t, reinterpret_cast<vu2_t *>(p));
      }
      return;
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e)
    if (e < valid) store_one(p + e, v[e]);
}

// One round in difference form, for the rows i of this block's group:
//   out[i,:] = cur[i,:] + c_mix * sum_k w[k] * (cur[col[k],:] - cur[i,:]) + eta * (cur[i,:] - prev[i,:])
// (= c_mix * (W^T cur)[i,:] - eta * prev[i,:] for c_mix = 1 + eta, the rows of W^T summing to one).  Written
// this way, equal values across the workers are reproduced exactly whatever the rounding of the weights, so
// the worker mean does not drift over many rounds; and the increment is formed at its own (small) magnitude,
// so the only rounding at the magnitude of the state is the last add.
// With HAS_G: out[i,:] = cur[i,:] + sum_k ... - alpha * G[i,:] (D-PSGD) and prev is not read.
template <typename ST, int VEC, bool HAS_G>
__global__ __launch_bounds__(kThreads) void gossip_round_kernel(int n, int64_t d, int64_t ld,
                                                                const int32_t *__restrict__ rowptr,
                                                                const int32_t *__restrict__ colidx,
                                                                const float *__restrict__ vals,
                                                                const ST *__restrict__ cur, const ST *prev, ST *out,
                                                                const float *__restrict__ G, float c_mix,
                                                                float eta, float alpha, int rows_per_group) {
  const int64_t c0 = (int64_t(blockIdx.x) * kThreads + threadIdx.x) * VEC;
  if (c0 >= d) return;
  const int valid = int(d - c0 < VEC ? d - c0 : VEC);
  const int r0 = blockIdx.y * rows_per_group;
  const int r1 = r0 + rows_per_group < n ? r0 + rows_per_group : n;
  for (int i = r0; i < r1; ++i) {
    float own[VEC], acc[VEC];
    load_vec<ST, VEC, false>(cur + int64_t(i) * ld + c0, valid, own);
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    const int k1 = rowptr[i + 1];
    for (int k = rowptr[i]; k < k1; ++k) {
      const int j = colidx[k];
      if (j == i) continue;  // the diagonal entry contributes a zero difference
      const float w = vals[k];
      float v[VEC];
      load_vec<ST, VEC, false>(cur + int64_t(j) * ld + c0, valid, v);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] = fmaf(w, v[e] - own[e], acc[e]);
    }
    float o[VEC];
    if constexpr (HAS_G) {
      float g[VEC];
      load_vec<float, VEC>(G + int64_t(i) * ld + c0, valid, g);
#pragma unroll
      for (int e = 0; e < VEC; ++e) o[e] = own[e] + fmaf(-alpha, g[e], c_mix * acc[e]);
    } else {
      float p[VEC];
      load_vec<ST, VEC>(prev + int64_t(i) * ld + c0, valid, p);
#pragma unroll
      for (int e = 0; e < VEC; ++e) o[e] = own[e] + fmaf(c_mix, acc[e], eta * (own[e] - p[e]));
    }
    store_vec<ST, VEC>(out + int64_t(i) * ld + c0, valid, o);
  }
}

// The same round with the neighbour tile staged in LDS, for n <= kTileRowsMax workers.  A block of kTileWaves
// wavefronts owns 64 columns and all n rows of them: row i of z_r is loaded once (wavefront i mod kTileWaves,
// 256 contiguous bytes), parked in LDS as fp32, and after one barrier every output row takes its neighbours from
// there.  HBM sees z_r once, z_{r-1} (or G) once and the output once: 12 bytes per element, where the kernel
// above re-fetches every row once per neighbour that reads it.  Row indices are uniform in a wavefront, so the
// CSR row (pointers, columns, weights) is read with scalar loads.  Every access goes through a buffer resource:
// the ragged last tile and odd pitches need no separate path.  The launcher takes this kernel for matrices of
// kTileMinBytes and more, with 4, 8 or 16 wavefronts per block for n <= 64, 128, 256 (about 16 rows per wavefront;
// fewer wavefronts keep too few loads in flight at large n).  Measured per round, fp32: 8x8 torus at 256 MiB
// 188 us against 236 us for the kernel above, at 1 GiB 696 against 960 us; random 4-regular graph, n = 256, 1 GiB:
// 750 against 1210 us.  Below about 128 MiB the caches serve the re-reads of the kernel above and it is the
// faster one (64 MiB: 46 against 53 us), so it keeps those.
constexpr int kTileCols = 64, kTileRowsMax = 256, kTileBatch = 4;
constexpr int64_t kTileMinBytes = int64_t(128) << 20;

template <typename ST, bool HAS_G, int kTileWaves>
__global__ __launch_bounds__(64 * kTileWaves) void gossip_round_tile_kernel(int n, int64_t d, int64_t ld,
                                                                         const int32_t *__restrict__ rowptr,
                                                                         const int32_t *__restrict__ colidx,
                                                                         const float *__restrict__ vals,
                                                                         const ST *cur, const ST *prev,
                                                                         ST *out, const float *__restrict__ G,
                                                                         float c_mix, float eta, float alpha) {
  extern __shared__ float tile_lds[];  // n x 64
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int64_t tile = int64_t(blockIdx.x) * kTileCols;
  const uint32_t valid = uint32_t(d - tile < kTileCols ? d - tile : kTileCols);
  const uint32_t so = lane * uint32_t(sizeof(ST)), fo = lane * 4u;
  for (int i0 = w; i0 < n; i0 += kTileWaves * kTileBatch) {
    float z[kTileBatch];
#pragma unroll
    for (int q = 0; q < kTileBatch; ++q) {
      const int i = i0 + q * kTileWaves;
      z[q] = buf_load<ST>(row_of(cur, tile, ld, i < n ? i : 0, i < n ? valid : 0u), so);
    }
#pragma unroll
    for (int q = 0; q < kTileBatch; ++q) {
      const int i = i0 + q * kTileWaves;
      if (i < n) tile_lds[i * kTileCols + lane] = z[q];
    }
  }
  __syncthreads();
  for (int i0 = w; i0 < n; i0 += kTileWaves * kTileBatch) {
    float other[kTileBatch];  // z_{r-1} (or the gradient) of this batch of rows, requested before the sums
#pragma unroll
    for (int q = 0; q < kTileBatch; ++q) {
      const int i = i0 + q * kTileWaves;
      if constexpr (HAS_G) other[q] = buf_load<float>(row_of(G, tile, ld, i < n ? i : 0, i < n ? valid : 0u), fo);
      else other[q] = buf_load<ST>(row_of(prev, tile, ld, i < n ? i : 0, i < n ? valid : 0u), so);
    }
#pragma unroll
    for (int q = 0; q < kTileBatch; ++q) {
      const int i = i0 + q * kTileWaves;
      if (i >= n) break;
      const float own = tile_lds[i * kTileCols + lane];
      float acc = 0.f;
      const int k1 = rowptr[i + 1];
      for (int k = rowptr[i]; k < k1; ++k) {
        const int j = colidx[k];
        acc = fmaf(vals[k], tile_lds[j * kTileCols + lane] - own, acc);  // j == i adds an exact zero
      }
      float o;
      if constexpr (HAS_G) o = own + fmaf(-alpha, other[q], c_mix * acc);
      else o = own + fmaf(c_mix, acc, eta * (own - other[q]));
      buf_store<ST>(row_of(out, tile, ld, i, valid), so, o);
    }
  }
}

// mode 0: Y += Gn - Go.   mode 1: X -= alpha*Y (Y before the update); Y += Gn - Go.
template <typename ST, int VEC, int MODE>
__global__ __launch_bounds__(kThreads) void elementwise_kernel(int64_t d, int64_t ld, ST *X, ST *Y,
                                                               const float *__restrict__ Gn,
                                                               const float *__restrict__ Go, float alpha) {
  const int64_t c0 = (int64_t(blockIdx.x) * kThreads + threadIdx.x) * VEC;
  if (c0 >= d) return;
  const int valid = int(d - c0 < VEC ? d - c0 : VEC);
  const int64_t off = int64_t(blockIdx.y) * ld + c0;
  float y[VEC], gn[VEC], go[VEC];
  load_vec<ST, VEC>(Y + off, valid, y);
  load_vec<float, VEC>(Gn + off, valid, gn);
  load_vec<float, VEC>(Go + off, valid, go);
  if constexpr (MODE == 1) {
    float x[VEC];
    load_vec<ST, VEC>(X + off, valid, x);
#pragma unroll
    for (int e = 0; e < VEC; ++e) x[e] = fmaf(-alpha, y[e], x[e]);
    store_vec<ST, VEC>(X + off, valid, x);
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) y[e] = y[e] + gn[e] - go[e];
  store_vec<ST, VEC>(Y + off, valid, y);
}

// out[i,:] = sum_k vals[k] * cur[col[k],:] for a general sparse matrix (rows need not sum to one, may be empty):
// the factor matrices of the exact average consensus (Lemma 1).
template <typename ST, int VEC>
__global__ __launch_bounds__(kThreads) void spmm_kernel(int n, int64_t d, int64_t ld, const int32_t *__restrict__ rowptr,
                                                        const int32_t *__restrict__ colidx,
                                                        const float *__restrict__ vals, const ST *__restrict__ cur,
                                                        ST *__restrict__ out, int rows_per_group) {
  const int64_t c0 = (int64_t(blockIdx.x) * kThreads + threadIdx.x) * VEC;
  if (c0 >= d) return;
  const int valid = int(d - c0 < VEC ? d - c0 : VEC);
  const int r0 = blockIdx.y * rows_per_group;
  const int r1 = r0 + rows_per_group < n ? r0 + rows_per_group : n;
  for (int i = r0; i < r1; ++i) {
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    const int k1 = rowptr[i + 1];
    for (int k = rowptr[i]; k < k1; ++k) {
      const float w = vals[k];
      float v[VEC];
      load_vec<ST, VEC, false>(cur + int64_t(colidx[k]) * ld + c0, valid, v);
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] = fmaf(w, v[e], acc[e]);
    }
    store_vec<ST, VEC>(out + int64_t(i) * ld + c0, valid, acc);
  }
}

// End of a round of Algorithm 1: X = Xt - scale*G; Xt = X; G = 0.
template <typename ST, int VEC>
__global__ __launch_bounds__(kThreads) void defacto_update_kernel(int64_t d, int64_t ld, ST *X, ST *Xt, float *G,
                                                                  float scale) {
  const int64_t c0 = (int64_t(blockIdx.x) * kThreads + threadIdx.x) * VEC;
  if (c0 >= d) return;
  const int valid = int(d - c0 < VEC ? d - c0 : VEC);
  const int64_t off = int64_t(blockIdx.y) * ld + c0;
  float x[VEC], g[VEC];
  load_vec<ST, VEC>(Xt + off, valid, x);
  load_vec<float, VEC>(G + off, valid, g);
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    x[e] = fmaf(-scale, g[e], x[e]);
    g[e] = 0.f;
  }
  store_vec<ST, VEC>(X + off, valid, x);
  if (Xt != X) store_vec<ST, VEC>(Xt + off, valid, x);
  store_vec<float, VEC>(G + off, valid, g);
}

// Gacc += scale * g
template <int VEC>
__global__ __launch_bounds__(kThreads) void accumulate_kernel(int64_t d, int64_t ld, float *Gacc,
                                                              const float *__restrict__ g, float scale) {
  const int64_t c0 = (int64_t(blockIdx.x) * kThreads + threadIdx.x) * VEC;
  if (c0 >= d) return;
  const int valid = int(d - c0 < VEC ? d - c0 : VEC);
  const int64_t off = int64_t(blockIdx.y) * ld + c0;
  float a[VEC], x[VEC];
  load_vec<float, VEC>(Gacc + off, valid, a);
  load_vec<float, VEC>(g + off, valid, x);
#pragma unroll
  for (int e = 0; e < VEC; ++e) a[e] = fmaf(scale, x[e], a[e]);
  store_vec<float, VEC>(Gacc + off, valid, a);
}

// End of a phase of Algorithm 2: X = Xt - alpha*Y; Y += Gk - Gkm1; Xt = X; Gkm1 = 0.
template <typename ST, int VEC>
__global__ __launch_bounds__(kThreads) void phase_end_kernel(int64_t d, int64_t ld, ST *X, ST *Xt, ST *Y,
                                                             const float *__restrict__ Gk, float *Gkm1, float alpha) {
  const int64_t c0 = (int64_t(blockIdx.x) * kThreads + threadIdx.x) * VEC;
  if (c0 >= d) return;
  const int valid = int(d - c0 < VEC ? d - c0 : VEC);
  const int64_t off = int64_t(blockIdx.y) * ld + c0;
  float x[VEC], y[VEC], gk[VEC], gm[VEC];
  load_vec<ST, VEC>(Xt + off, valid, x);
  load_vec<ST, VEC>(Y + off, valid, y);
  load_vec<float, VEC>(Gk + off, valid, gk);
  load_vec<float, VEC>(Gkm1 + off, valid, gm);
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    x[e] = fmaf(-alpha, y[e], x[e]);
    y[e] = y[e] + gk[e] - gm[e];
    gm[e] = 0.f;
  }
  store_vec<ST, VEC>(X + off, valid, x);
  if (Xt != X) store_vec<ST, VEC>(Xt + off, valid, x);
  store_vec<ST, VEC>(Y + off, valid, y);
  store_vec<float, VEC>(Gkm1 + off, valid, gm);
}

// dst = src with a change of storage type (bf16 -> fp32 exact, fp32 -> bf16 round to nearest even)
template <typename TS, typename TD, int VEC>
__global__ __launch_bounds__(kThreads) void convert_kernel(int64_t d, int64_t ld, const TS *__restrict__ src,
                                                           TD *__restrict__ dst) {
  const int64_t c0 = (int64_t(blockIdx.x) * kThreads + threadIdx.x) * VEC;
  if (c0 >= d) return;
  const int valid = int(d - c0 < VEC ? d - c0 : VEC);
  const int64_t off = int64_t(blockIdx.y) * ld + c0;
  float x[VEC];
  load_vec<TS, VEC>(src + off, valid, x);
  store_vec<TD, VEC>(dst + off, valid, x);
}

// 16-byte accesses need every row start 16-byte aligned (8 bytes for bf16 vectors of four).
bool vec_ok(const Shape &s, std::initializer_list<const void *> state_ptrs, std::initializer_list<const void *> f32_ptrs) {
  if (s.ld % 4) return false;
  const uintptr_t smask = s.bf16 ? 7 : 15;
  for (const void *p : state_ptrs)
    if (p && (reinterpret_cast<uintptr_t>(p) & smask)) return false;
  for (const void *p : f32_ptrs)
    if (p && (reinterpret_cast<uintptr_t>(p) & 15)) return false;
  return true;
}

int rows_per_group_for(const Shape &s, int col_blocks) {
  // Enough blocks to fill 256 CUs several times over; one group (all rows in one
  // block, neighbour re-reads stay in that CU's caches) once columns alone do it.
  if (col_blocks >= 2048) return s.n;
  int groups = (2048 + col_blocks - 1) / col_blocks;
  if (groups > s.n) groups = s.n;
  return (s.n + groups - 1) / groups;
}

template <typename ST, bool HAS_G>
int launch_round_t(const Shape &s, const DevCsr &w, const void *cur, const void *prev, void *out, const float *G,
                   float c_mix, float eta, float alpha, void *stream) {
  auto st = static_cast<hipStream_t>(stream);
  if (round_stages_tile(s)) {
    const dim3 tgrid(ceil_div_i64(s.d, kTileCols));
    const size_t lds_bytes = size_t(s.n) * kTileCols * sizeof(float);
#define DETAG_TILE_GO(RW)                                                                                      \
  gossip_round_tile_kernel<ST, HAS_G, RW><<<tgrid, 64 * RW, lds_bytes, st>>>(                                  \
      s.n, s.d, s.ld, w.rowptr, w.colidx, w.vals, static_cast<const ST *>(cur), static_cast<const ST *>(prev), \
      static_cast<ST *>(out), G, c_mix, eta, alpha)
    if (s.n <= 64) DETAG_TILE_GO(4);
    else if (s.n <= 128) DETAG_TILE_GO(8);
    else DETAG_TILE_GO(16);
#undef DETAG_TILE_GO
    return hip_rc(hipGetLastError());
  }
  const bool vec = vec_ok(s, {cur, prev, out}, {G});
  const int per_block = kThreads * (vec ? 4 : 1);
  const int col_blocks = ceil_div_i64(s.d, per_block);
  const int rpg = rows_per_group_for(s, col_blocks);
  dim3 grid(col_blocks, (s.n + rpg - 1) / rpg);
  if (vec)
    gossip_round_kernel<ST, 4, HAS_G><<<grid, kThreads, 0, st>>>(
        s.n, s.d, s.ld, w.rowptr, w.colidx, w.vals, static_cast<const ST *>(cur), static_cast<const ST *>(prev),
        static_cast<ST *>(out), G, c_mix, eta, alpha, rpg);
  else
    gossip_round_kernel<ST, 1, HAS_G><<<grid, kThreads, 0, st>>>(
        s.n, s.d, s.ld, w.rowptr, w.colidx, w.vals, static_cast<const ST *>(cur), static_cast<const ST *>(prev),
        static_cast<ST *>(out), G, c_mix, eta, alpha, rpg);
  return hip_rc(hipGetLastError());
}

template <typename ST, int MODE>
int launch_elementwise_t(const Shape &s, void *X, void *Y, const float *Gn, const float *Go, float alpha,
                         void *stream) {
  const bool vec = vec_ok(s, {X, Y}, {Gn, Go});
  const int per_block = kThreads * (vec ? 4 : 1);
  dim3 grid(ceil_div_i64(s.d, per_block), s.n);
  auto st = static_cast<hipStream_t>(stream);
  if (vec)
    elementwise_kernel<ST, 4, MODE><<<grid, kThreads, 0, st>>>(s.d, s.ld, static_cast<ST *>(X),
                                                                static_cast<ST *>(Y), Gn, Go, alpha);
  else
    elementwise_kernel<ST, 1, MODE><<<grid, kThreads, 0, st>>>(s.d, s.ld, static_cast<ST *>(X),
                                                                static_cast<ST *>(Y), Gn, Go, alpha);
  return hip_rc(hipGetLastError());
}

template <typename TS, typename TD>
int launch_convert_t(const Shape &s, const void *src, void *dst, void *stream) {
  const bool vec = s.ld % 4 == 0 && (reinterpret_cast<uintptr_t>(src) % (4 * sizeof(TS))) == 0 &&
                   (reinterpret_cast<uintptr_t>(dst) % (4 * sizeof(TD))) == 0;
  dim3 grid(ceil_div_i64(s.d, kThreads * (vec ? 4 : 1)), s.n);
  auto st = static_cast<hipStream_t>(stream);
  if (vec)
    convert_kernel<TS, TD, 4><<<grid, kThreads, 0, st>>>(s.d, s.ld, static_cast<const TS *>(src),
                                                         static_cast<TD *>(dst));
  else
    convert_kernel<TS, TD, 1><<<grid, kThreads, 0, st>>>(s.d, s.ld, static_cast<const TS *>(src),
                                                         static_cast<TD *>(dst));
  return hip_rc(hipGetLastError());
}

}  // namespace

template <typename ST>
int launch_spmm_t(const Shape &s, const DevCsr &a, const void *cur, void *out, void *stream) {
  const bool vec = vec_ok(s, {cur, out}, {});
  const int col_blocks = ceil_div_i64(s.d, kThreads * (vec ? 4 : 1));
  const int rpg = rows_per_group_for(s, col_blocks);
  dim3 grid(col_blocks, (s.n + rpg - 1) / rpg);
  auto st = static_cast<hipStream_t>(stream);
  if (vec)
    spmm_kernel<ST, 4><<<grid, kThreads, 0, st>>>(s.n, s.d, s.ld, a.rowptr, a.colidx, a.vals,
                                                  static_cast<const ST *>(cur), static_cast<ST *>(out), rpg);
  else
    spmm_kernel<ST, 1><<<grid, kThreads, 0, st>>>(s.n, s.d, s.ld, a.rowptr, a.colidx, a.vals,
                                                  static_cast<const ST *>(cur), static_cast<ST *>(out), rpg);
  return hip_rc(hipGetLastError());
}

int launch_spmm(const Shape &s, const DevCsr &a, const void *cur, void *out, void *stream) {
  return s.bf16 ? launch_spmm_t<bf16_t>(s, a, cur, out, stream) : launch_spmm_t<float>(s, a, cur, out, stream);
}

template <typename ST>
int launch_defacto_update_t(const Shape &s, void *X, void *Xt, float *G, float scale, void *stream) {
  const bool vec = vec_ok(s, {X, Xt}, {G});
  dim3 grid(ceil_div_i64(s.d, kThreads * (vec ? 4 : 1)), s.n);
  auto st = static_cast<hipStream_t>(stream);
  if (vec)
    defacto_update_kernel<ST, 4><<<grid, kThreads, 0, st>>>(s.d, s.ld, static_cast<ST *>(X), static_cast<ST *>(Xt), G,
                                                            scale);
  else
    defacto_update_kernel<ST, 1><<<grid, kThreads, 0, st>>>(s.d, s.ld, static_cast<ST *>(X), static_cast<ST *>(Xt), G,
                                                            scale);
  return hip_rc(hipGetLastError());
}

int launch_defacto_update(const Shape &s, void *X, void *Xt, float *G, float scale, void *stream) {
  return s.bf16 ? launch_defacto_update_t<bf16_t>(s, X, Xt, G, scale, stream)
                : launch_defacto_update_t<float>(s, X, Xt, G, scale, stream);
}

int launch_accumulate(const Shape &s, float *Gacc, const float *g, float scale, void *stream) {
  const bool vec = vec_ok(s, {}, {Gacc, g});
  dim3 grid(ceil_div_i64(s.d, kThreads * (vec ? 4 : 1)), s.n);
  auto st = static_cast<hipStream_t>(stream);
  if (vec) accumulate_kernel<4><<<grid, kThreads, 0, st>>>(s.d, s.ld, Gacc, g, scale);
  else accumulate_kernel<1><<<grid, kThreads, 0, st>>>(s.d, s.ld, Gacc, g, scale);
  return hip_rc(hipGetLastError());
}

template <typename ST>
int launch_phase_end_t(const Shape &s, void *X, void *Xt, void *Y, const float *Gk, float *Gkm1, float alpha,
                       void *stream) {
  const bool vec = vec_ok(s, {X, Xt, Y}, {Gk, Gkm1});
  dim3 grid(ceil_div_i64(s.d, kThreads * (vec ? 4 : 1)), s.n);
  auto st = static_cast<hipStream_t>(stream);
  if (vec)
    phase_end_kernel<ST, 4><<<grid, kThreads, 0, st>>>(s.d, s.ld, static_cast<ST *>(X), static_cast<ST *>(Xt),
                                                       static_cast<ST *>(Y), Gk, Gkm1, alpha);
  else
    phase_end_kernel<ST, 1><<<grid, kThreads, 0, st>>>(s.d, s.ld, static_cast<ST *>(X), static_cast<ST *>(Xt),
                                                       static_cast<ST *>(Y), Gk, Gkm1, alpha);
  return hip_rc(hipGetLastError());
}

int launch_phase_end(const Shape &s, void *X, void *Xt, void *Y, const float *Gk, float *Gkm1, float alpha,
                     void *stream) {
  return s.bf16 ? launch_phase_end_t<bf16_t>(s, X, Xt, Y, Gk, Gkm1, alpha, stream)
                : launch_phase_end_t<float>(s, X, Xt, Y, Gk, Gkm1, alpha, stream);
}

int launch_widen(const Shape &s, const void *src_bf16, float *dst, void *stream) {
  return launch_convert_t<bf16_t, float>(s, src_bf16, dst, stream);
}

int launch_narrow(const Shape &s, const float *src, void *dst_bf16, void *stream) {
  return launch_convert_t<float, bf16_t>(s, src, dst_bf16, stream);
}

// Whether a round on this shape takes the LDS-staged tile kernel.  That kernel reads all n rows of a column tile
// before it writes any, so its output may also be written over z_r itself (detag_dpsgd_step then needs no copy).
bool round_stages_tile(const Shape &s) {
  return s.n <= kTileRowsMax && int64_t(s.n) * s.ld * int64_t(s.bf16 ? 2 : 4) >= kTileMinBytes;
}

int launch_gossip_round(const Shape &s, const DevCsr &w, const void *cur, const void *prev, void *out, float eta,
                        void *stream) {
  return s.bf16 ? launch_round_t<bf16_t, false>(s, w, cur, prev, out, nullptr, 1.f + eta, eta, 0.f, stream)
                : launch_round_t<float, false>(s, w, cur, prev, out, nullptr, 1.f + eta, eta, 0.f, stream);
}

int launch_dpsgd(const Shape &s, const DevCsr &w, const void *Xin, void *X, const float *G, float alpha,
                 void *stream) {
  return s.bf16 ? launch_round_t<bf16_t, true>(s, w, Xin, nullptr, X, G, 1.f, 0.f, alpha, stream)
                : launch_round_t<float, true>(s, w, Xin, nullptr, X, G, 1.f, 0.f, alpha, stream);
}

int launch_track(const Shape &s, void *Y, const float *Gn, const float *Go, void *stream) {
  return s.bf16 ? launch_elementwise_t<bf16_t, 0>(s, nullptr, Y, Gn, Go, 0.f, stream)
                : launch_elementwise_t<float, 0>(s, nullptr, Y, Gn, Go, 0.f, stream);
}

int launch_update_track(const Shape &s, void *X, void *Y, const float *Gn, const float *Go, float alpha,
                        void *stream) {
  return s.bf16 ? launch_elementwise_t<bf16_t, 1>(s, X, Y, Gn, Go, alpha, stream)
                : launch_elementwise_t<float, 1>(s, X, Y, Gn, Go, alpha, stream);
}

int launch_copy_state(const Shape &s, const void *src, void *dst, void *stream) {
  return s.bf16 ? launch_convert_t<bf16_t, bf16_t>(s, src, dst, stream) : launch_convert_t<float, float>(s, src, dst, stream);
}

}  // namespace detag
