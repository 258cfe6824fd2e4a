// C ABI of the DeTAG hot path (see include/detag.h): argument checks, the
// context, and the order in which kernels are enqueued.  No arithmetic of the
// method happens on the host after detag_create.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>

#include "detag_internal.h"

using namespace detag;

struct detag_ctx {
  HostW W;
  Shape shape{};
  bool has_device = false;
  int device = -1;
  int32_t *d_rowptr = nullptr, *d_colidx = nullptr;
  float *d_vals = nullptr;
  uint32_t *d_ell_table = nullptr;  // neighbour table of the on-chip kernel for arbitrary W
  int ell_deg = 0;
  bool ell_uniform = false;
  bool fused_generic = false;             // build_ell succeeded for this W
  // per-round path: n x ld fp32 matrices; [0],[1] hold z_r between rounds, [2],[3] the widened copies of bf16 X and Y
  void *scratch[4] = {nullptr, nullptr, nullptr, nullptr};
  double *d_partials = nullptr;           // consensus-error partial sums
  float *d_resid = nullptr;               // gradient scratch: least-squares residuals / softmax residuals
  int64_t resid_count = 0;
  detag_path path = DETAG_PATH_AUTO;
  // DETAG_PATH_DENSE: the last few polynomials p_K(W^T) on the device
  struct DensePoly {
    int K = -1;
    float eta = 0.f;
    uint16_t *d_frag = nullptr;
    uint64_t used = 0;
  };
  DensePoly poly[4];
  uint64_t poly_clock = 0;
  mutable std::string err;
};

struct detag_factors {
  detag_ctx *ctx = nullptr;
  std::vector<HostFactor> host;
  // device copies, all factors back to back: rowptr R*(n+1), colidx / vals at offs[r]
  int32_t *d_rowptr = nullptr, *d_colidx = nullptr;
  float *d_vals = nullptr;
  std::vector<int64_t> offs;
  std::vector<uint32_t> table;  // program of the on-chip kernel; empty if build_factor_table declined
  uint32_t *d_table = nullptr;
};

namespace {

thread_local std::string g_create_err;

detag_status set_err(const detag_ctx *ctx, detag_status st, const std::string &msg) {
  if (ctx) ctx->err = msg; else g_create_err = msg;
  return st;
}

detag_status hip_fail(const detag_ctx *ctx, const char *what, int rc) {
  char buf[256];
  std::snprintf(buf, sizeof buf, "%s: %s", what, hipGetErrorString(static_cast<hipError_t>(rc)));
  return set_err(ctx, DETAG_EHIP, buf);
}

size_t scratch_bytes(const Shape &s) { return size_t(s.n) * size_t(s.ld) * 4; }  // fp32 whatever the state type

detag_status need_device(const detag_ctx *ctx) {
  if (!ctx) return DETAG_EINVAL;
  if (!ctx->has_device) return set_err(ctx, DETAG_EHIP, "no GPU was present when this context was created");
  return DETAG_OK;
}

// A stream that is being recorded into a HIP graph must see kernel launches only: an allocation, a blocking
// copy or a device synchronisation would fail or invalidate the recording half-way.
bool is_capturing(void *stream) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(static_cast<hipStream_t>(stream), &st) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return st != hipStreamCaptureStatusNone;
}

detag_status refuse_while_capturing(const detag_ctx *ctx, const char *what, const char *reserve) {
  return set_err(ctx, DETAG_EINVAL, std::string("the stream is being captured and this call would have to allocate ") +
                                        what + ": call " + reserve + " before the capture begins");
}

detag_status need_scratch(detag_ctx *ctx, int first, int count, void *stream) {
  for (int k = first; k < first + count; ++k)
    if (!ctx->scratch[k]) {
      if (is_capturing(stream)) return refuse_while_capturing(ctx, "the per-round gossip scratch", "detag_reserve_gossip");
      hipError_t e = hipMalloc(&ctx->scratch[k], scratch_bytes(ctx->shape));
      if (e != hipSuccess) {
        ctx->scratch[k] = nullptr;
        (void)hipGetLastError();
        return set_err(ctx, DETAG_ENOMEM, "could not allocate the per-round gossip scratch");
      }
    }
  return DETAG_OK;
}

detag_status need_grad_scratch(detag_ctx *ctx, int64_t floats, void *stream) {
  if (ctx->resid_count >= floats) return DETAG_OK;
  if (is_capturing(stream)) return refuse_while_capturing(ctx, "the gradient scratch", "detag_reserve_gradient");
  (void)hipFree(ctx->d_resid);
  ctx->d_resid = nullptr, ctx->resid_count = 0;
  if (hipMalloc(reinterpret_cast<void **>(&ctx->d_resid), size_t(floats) * sizeof(float)) != hipSuccess) {
    (void)hipGetLastError();
    return set_err(ctx, DETAG_ENOMEM, "could not allocate the gradient scratch");
  }
  ctx->resid_count = floats;
  return DETAG_OK;
}

bool misaligned(const void *p, size_t a) { return reinterpret_cast<uintptr_t>(p) % a != 0; }

detag_status resolve_eta(const detag_ctx *ctx, double eta_in, float *eta_out) {
  double eta = eta_in;
  if (eta < 0) {
    eta = ctx->W.eta;
    if (std::isnan(eta))
      return set_err(ctx, DETAG_EINVAL, "W is not symmetric, so it has no stored eta: pass eta explicitly");
  }
  if (!(eta >= 0.0 && eta < 1.0)) return set_err(ctx, DETAG_EINVAL, "eta must be in [0, 1)");
  *eta_out = float(eta);
  return DETAG_OK;
}

DevCsr dev_csr(const detag_ctx *ctx) {
  DevCsr w;
  w.rowptr = ctx->d_rowptr, w.colidx = ctx->d_colidx, w.vals = ctx->d_vals;
  w.ell_table = ctx->d_ell_table, w.ell_deg = ctx->ell_deg, w.ell_uniform = ctx->ell_uniform;
  return w;
}

enum Chosen { kPerRound, kFusedStructured, kFusedGeneric, kDense };

detag_status choose_path(const detag_ctx *ctx, Chosen *out) {
  const bool fs = fused_structured_available(ctx->W), fg = ctx->fused_generic;
  if (ctx->path == DETAG_PATH_PER_ROUND) return *out = kPerRound, DETAG_OK;
  if (ctx->path == DETAG_PATH_DENSE) return *out = kDense, DETAG_OK;
  if (fs) return *out = kFusedStructured, DETAG_OK;
  if (fg) return *out = kFusedGeneric, DETAG_OK;
  if (ctx->path == DETAG_PATH_FUSED)
    return set_err(ctx, DETAG_EUNSUPPORTED, "no fused kernel for this topology and n");
  return *out = kPerRound, DETAG_OK;
}

Shape as_f32(Shape s) { return s.bf16 = false, s; }

// The device copy of p_K(W^T) for DETAG_PATH_DENSE: from the context's small cache, or evaluated and uploaded now.
// A buffer is rewritten only after the device has drained, since an earlier launch may still read it.
detag_status dense_poly(detag_ctx *ctx, int K, float eta, const uint16_t **frag, void *stream) {
  detag_ctx::DensePoly *slot = nullptr;
  for (auto &e : ctx->poly)
    if (e.d_frag && e.K == K && e.eta == eta) slot = &e;
  if (!slot) {
    if (is_capturing(stream))
      return refuse_while_capturing(ctx, "and upload the gossip polynomial of this (K, eta)", "detag_reserve_gossip");
    const int terms = dense_poly_terms(ctx->shape.bf16);
    std::vector<uint16_t> host;
    if (!build_dense_poly(ctx->W, K, double(eta), terms, host))
      return set_err(ctx, DETAG_EUNSUPPORTED, "the dense path needs n <= 256");
    for (auto &e : ctx->poly)
      if (!slot || e.used < slot->used) slot = &e;  // least recently used (unused slots have used == 0)
    hipError_t err = hipSuccess;
    if (slot->d_frag) err = hipDeviceSynchronize();
    else err = hipMalloc(reinterpret_cast<void **>(&slot->d_frag), host.size() * sizeof(uint16_t));
    if (err == hipSuccess) err = hipMemcpy(slot->d_frag, host.data(), host.size() * sizeof(uint16_t), hipMemcpyHostToDevice);
    if (err != hipSuccess) {
      slot->K = -1;
      return hip_fail(ctx, "uploading the gossip polynomial", int(err));
    }
    slot->K = K, slot->eta = eta;
  }
  slot->used = ++ctx->poly_clock;
  *frag = slot->d_frag;
  return DETAG_OK;
}

// One round with z_{r-1} given.  Ring and torus contexts with a register-resident kernel take that family's
// one-round kernel (every row read once, 12 B per element; measured as fast as or faster than the CSR kernels at
// every size from 1 MiB up: 34 against 46 us per round at 64 MiB); everything else the CSR kernels (LDS-staged
// from 128 MiB on, cache-served below).
int round_launch(const detag_ctx *ctx, const Shape &s, const void *cur, const void *prev, void *out, float eta,
                 void *stream) {
  if (fused_structured_available(ctx->W))
    return launch_structured_round(s, ctx->W, cur, prev, out, eta, stream);
  return launch_gossip_round(s, dev_csr(ctx), cur, prev, out, eta, stream);
}

// Algorithm 3 with one launch per round on an fp32 matrix A.  z_r lives in A or
// in scratch; a round may write over its own z_{r-1} (each output element reads
// only its own previous value) but never over z_r, which every neighbour reads.
detag_status gossip_per_round_f32(detag_ctx *ctx, void *A, int K, float eta, void *stream) {
  if (K == 0) return DETAG_OK;
  const int nscratch = (K % 2 == 1 && K >= 3) ? 2 : 1;
  if (detag_status st = need_scratch(ctx, 0, nscratch, stream)) return st;
  void *B = ctx->scratch[0], *C = ctx->scratch[1];
  const Shape s = as_f32(ctx->shape);
  int rc = round_launch(ctx, s, A, A, B, eta, stream);  // z1 -> B
  if (rc) return hip_fail(ctx, "gossip round", rc);
  if (K == 1) {
    rc = launch_copy_state(s, B, A, stream);
    return rc ? hip_fail(ctx, "copy", rc) : DETAG_OK;
  }
  int r = 1;           // next round computes z_{r+1}
  void *cur = B, *prev = A;
  if (K % 2 == 1) {    // shift parity once through the third buffer: z2 -> C, z3 -> A
    rc = round_launch(ctx, s, B, A, C, eta, stream);
    if (!rc) rc = round_launch(ctx, s, C, B, A, eta, stream);
    if (rc) return hip_fail(ctx, "gossip round", rc);
    r = 3, cur = A, prev = C;
  }
  for (; r < K; ++r) {  // z_{r+1} overwrites z_{r-1}
    rc = round_launch(ctx, s, cur, prev, prev, eta, stream);
    if (rc) return hip_fail(ctx, "gossip round", rc);
    void *t = cur; cur = prev; prev = t;
  }
  if (cur != A) return set_err(ctx, DETAG_EHIP, "internal: gossip result not in the caller's buffer");
  return DETAG_OK;
}

// The per-round path computes on fp32 matrices.  bf16 state is widened into
// scratch once (exact), worked on there, and rounded once when it is written
// back, so this path and the on-chip kernels round the same number of times.
struct WideState {
  detag_ctx *ctx;
  void *user[2] = {nullptr, nullptr};
  void *work[2] = {nullptr, nullptr};

  detag_status open(void *a, void *b, void *stream) {
    user[0] = a, user[1] = b;
    work[0] = a, work[1] = b;
    if (!ctx->shape.bf16) return DETAG_OK;
    if (detag_status st = need_scratch(ctx, 2, b ? 2 : 1, stream)) return st;
    for (int k = 0; k < 2 && user[k]; ++k) {
      work[k] = ctx->scratch[2 + k];
      if (int rc = launch_widen(ctx->shape, user[k], static_cast<float *>(work[k]), stream))
        return hip_fail(ctx, "widen", rc);
    }
    return DETAG_OK;
  }
  detag_status close(void *stream) {
    if (!ctx->shape.bf16) return DETAG_OK;
    for (int k = 0; k < 2 && user[k]; ++k)
      if (int rc = launch_narrow(ctx->shape, static_cast<const float *>(work[k]), user[k], stream))
        return hip_fail(ctx, "narrow", rc);
    return DETAG_OK;
  }
};

detag_status check_state_ptr(const detag_ctx *ctx, const void *p, const char *name) {
  if (!p) return set_err(ctx, DETAG_EINVAL, std::string(name) + " is NULL");
  if (misaligned(p, ctx->shape.bf16 ? 2 : 4)) return set_err(ctx, DETAG_EINVAL, std::string(name) + " is misaligned");
  return DETAG_OK;
}

detag_status check_f32_ptr(const detag_ctx *ctx, const void *p, const char *name) {
  if (!p) return set_err(ctx, DETAG_EINVAL, std::string(name) + " is NULL");
  if (misaligned(p, 4)) return set_err(ctx, DETAG_EINVAL, std::string(name) + " is misaligned");
  return DETAG_OK;
}

}  // namespace

extern "C" {

detag_status detag_create(const detag_topology *topo, int32_t n, int64_t d, int64_t ld, int32_t state,
                          detag_ctx **out) {
  if (!out) return set_err(nullptr, DETAG_EINVAL, "out is NULL");
  *out = nullptr;
  if (n < 1 || n > 65535) return set_err(nullptr, DETAG_EINVAL, "n must be in [1, 65535]");
  if (d < 1) return set_err(nullptr, DETAG_EINVAL, "d must be >= 1");
  if (ld < d) return set_err(nullptr, DETAG_EINVAL, "ld must be >= d");
  if (state != DETAG_F32 && state != DETAG_BF16) return set_err(nullptr, DETAG_EINVAL, "unknown state dtype");
  detag_ctx *ctx = new (std::nothrow) detag_ctx();
  if (!ctx) return set_err(nullptr, DETAG_ENOMEM, "out of host memory");
  std::string err;
  detag_status st;
  try {
    st = build_gossip_matrix(topo, n, ctx->W, err);
  } catch (const std::bad_alloc &) {
    st = DETAG_ENOMEM, err = "out of host memory";
  }
  if (st != DETAG_OK) {
    delete ctx;
    return set_err(nullptr, st, err);
  }
  ctx->shape.n = n, ctx->shape.d = d, ctx->shape.ld = ld, ctx->shape.bf16 = state == DETAG_BF16;

  EllHost ell;
  ctx->fused_generic = build_ell(ctx->W, ell);

  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || count < 1) {
    (void)hipGetLastError();
    ctx->has_device = false;
    *out = ctx;
    return DETAG_OK;
  }
  ctx->has_device = true;
  (void)hipGetDevice(&ctx->device);
  // address of the library-resident partial sums on this device (detag_consensus_error_static); a failure is
  // reported by that entry point, which looks the address up again
  if (static_partials_init(ctx->device) != 0) (void)hipGetLastError();
  const size_t nnz = ctx->W.colidx.size();
  std::vector<float> vals32(nnz);
  for (size_t k = 0; k < nnz; ++k) vals32[k] = float(ctx->W.vals[k]);
  hipError_t e = hipMalloc(reinterpret_cast<void **>(&ctx->d_rowptr), (size_t(n) + 1) * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&ctx->d_colidx), nnz * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&ctx->d_vals), nnz * sizeof(float));
  if (e == hipSuccess)
    e = hipMalloc(reinterpret_cast<void **>(&ctx->d_partials), size_t(consensus_partials_count(ctx->shape)) * sizeof(double));
  if (e == hipSuccess)
    e = hipMemcpy(ctx->d_rowptr, ctx->W.rowptr.data(), (size_t(n) + 1) * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(ctx->d_colidx, ctx->W.colidx.data(), nnz * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(ctx->d_vals, vals32.data(), nnz * sizeof(float), hipMemcpyHostToDevice);
  if (ctx->fused_generic) {
    ctx->ell_deg = ell.deg, ctx->ell_uniform = ell.uniform;
    const size_t bytes = ell.table.size() * sizeof(uint32_t);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&ctx->d_ell_table), bytes);
    if (e == hipSuccess) e = hipMemcpy(ctx->d_ell_table, ell.table.data(), bytes, hipMemcpyHostToDevice);
  }
  if (e != hipSuccess) {
    const int rc = int(e);
    detag_destroy(ctx);
    return hip_fail(nullptr, "uploading the gossip matrix", rc);
  }
  *out = ctx;
  return DETAG_OK;
}

void detag_destroy(detag_ctx *ctx) {
  if (!ctx) return;
  if (ctx->has_device) {
    (void)hipDeviceSynchronize();
    (void)hipFree(ctx->d_rowptr);
    (void)hipFree(ctx->d_colidx);
    (void)hipFree(ctx->d_vals);
    (void)hipFree(ctx->d_ell_table);
    (void)hipFree(ctx->d_partials);
    (void)hipFree(ctx->d_resid);
    for (void *p : ctx->scratch) (void)hipFree(p);
    for (auto &e : ctx->poly) (void)hipFree(e.d_frag);
  }
  delete ctx;
}

detag_status detag_get_spectrum(const detag_ctx *ctx, double *lambda2, double *lambdan, double *lambda, double *eta) {
  if (!ctx) return set_err(nullptr, DETAG_EINVAL, "ctx is NULL");
  if (lambda2) *lambda2 = ctx->W.lambda2;
  if (lambdan) *lambdan = ctx->W.lambdan;
  if (lambda) *lambda = ctx->W.lambda;
  if (eta) *eta = ctx->W.eta;
  return DETAG_OK;
}

detag_status detag_get_phase_length(const detag_ctx *ctx, double outer_ratio, int32_t *R) {
  if (!ctx) return set_err(nullptr, DETAG_EINVAL, "ctx is NULL");
  if (!R) return set_err(ctx, DETAG_EINVAL, "R is NULL");
  const double lam = ctx->W.lambda;
  if (std::isnan(lam)) return set_err(ctx, DETAG_EINVAL, "W is not symmetric, so it has no stored lambda");
  if (std::isnan(outer_ratio)) return set_err(ctx, DETAG_EINVAL, "outer_ratio is NaN");
  double lead = 0.5 * std::log(double(ctx->W.n));
  if (outer_ratio > 0.0) lead = std::max(lead, 0.5 * std::log(outer_ratio));
  const double r = std::ceil(lead / std::sqrt(1.0 - lam));
  if (!(r < 2147483647.0)) return set_err(ctx, DETAG_EINVAL, "phase length does not fit an int32");
  *R = r < 1.0 ? 1 : int32_t(r);
  return DETAG_OK;
}

detag_status detag_get_csr(const detag_ctx *ctx, int32_t *n, int64_t *nnz, const int32_t **rowptr,
                           const int32_t **colidx, const double **vals) {
  if (!ctx) return set_err(nullptr, DETAG_EINVAL, "ctx is NULL");
  if (n) *n = ctx->W.n;
  if (nnz) *nnz = int64_t(ctx->W.colidx.size());
  if (rowptr) *rowptr = ctx->W.rowptr.data();
  if (colidx) *colidx = ctx->W.colidx.data();
  if (vals) *vals = ctx->W.vals.data();
  return DETAG_OK;
}

detag_status detag_set_path(detag_ctx *ctx, int32_t path) {
  if (!ctx) return set_err(nullptr, DETAG_EINVAL, "ctx is NULL");
  if (path != DETAG_PATH_AUTO && path != DETAG_PATH_PER_ROUND && path != DETAG_PATH_FUSED && path != DETAG_PATH_DENSE)
    return set_err(ctx, DETAG_EINVAL, "unknown path");
  if (path == DETAG_PATH_DENSE && ctx->W.n > 256)
    return set_err(ctx, DETAG_EUNSUPPORTED, "the dense path needs n <= 256");
  if (path == DETAG_PATH_FUSED && !detag_has_fused(ctx))
    return set_err(ctx, DETAG_EUNSUPPORTED, "no fused kernel for this topology and n");
  ctx->path = static_cast<detag_path>(path);
  return DETAG_OK;
}

detag_status detag_get_kernel(const detag_ctx *ctx, int32_t *kernel) {
  if (!ctx) return set_err(nullptr, DETAG_EINVAL, "ctx is NULL");
  if (!kernel) return set_err(ctx, DETAG_EINVAL, "kernel is NULL");
  Chosen c;
  if (detag_status st = choose_path(ctx, &c)) return st;
  *kernel = c == kFusedStructured ? DETAG_KERNEL_REGISTER_TILE
          : c == kFusedGeneric    ? DETAG_KERNEL_LDS_TILE
          : c == kDense           ? DETAG_KERNEL_DENSE
                                  : DETAG_KERNEL_PER_ROUND;
  return DETAG_OK;
}

int32_t detag_has_fused(const detag_ctx *ctx) {
  if (!ctx) return 0;
  return fused_structured_available(ctx->W) || ctx->fused_generic ? 1 : 0;
}

detag_status detag_get_gossip_polynomial(const detag_ctx *ctx, int32_t K, double eta, double *P_out) {
  if (!ctx) return set_err(nullptr, DETAG_EINVAL, "ctx is NULL");
  if (!P_out) return set_err(ctx, DETAG_EINVAL, "P_out is NULL");
  if (K < 0) return set_err(ctx, DETAG_EINVAL, "K must be >= 0");
  float e;
  if (detag_status st = resolve_eta(ctx, eta, &e)) return st;
  std::vector<double> P;
  try {
    gossip_polynomial(ctx->W, K, eta < 0 ? ctx->W.eta : eta, P);
  } catch (const std::bad_alloc &) {
    return set_err(ctx, DETAG_ENOMEM, "out of host memory");
  }
  std::copy(P.begin(), P.end(), P_out);
  return DETAG_OK;
}

detag_status detag_reserve_gossip(detag_ctx *ctx, int32_t path, int32_t K, double eta) {
  if (detag_status st = need_device(ctx)) return st;
  if (path != DETAG_PATH_PER_ROUND && path != DETAG_PATH_DENSE)
    return set_err(ctx, DETAG_EINVAL, "only DETAG_PATH_PER_ROUND and DETAG_PATH_DENSE own memory to reserve");
  if (path == DETAG_PATH_PER_ROUND)  // z_r buffers, and the widened copies of bf16 X and Y
    return need_scratch(ctx, 0, ctx->shape.bf16 ? 4 : 2, nullptr);
  if (ctx->W.n > 256) return set_err(ctx, DETAG_EUNSUPPORTED, "the dense path needs n <= 256");
  if (K < 1) return set_err(ctx, DETAG_EINVAL, "K must be >= 1");
  float e;
  if (detag_status st = resolve_eta(ctx, eta, &e)) return st;
  const uint16_t *frag = nullptr;
  return dense_poly(ctx, K, e, &frag, nullptr);
}

detag_status detag_reserve_gradient(detag_ctx *ctx, int32_t m, int32_t F, int32_t C, int32_t B) {
  if (detag_status st = need_device(ctx)) return st;
  if (m < 0 || F < 0 || C < 0 || B < 0) return set_err(ctx, DETAG_EINVAL, "sizes must be >= 0");
  int64_t floats = int64_t(ctx->shape.n) * m;
  if (F > 0 && C > 0 && B > 0) floats = std::max(floats, softmax_scratch_floats(ctx->shape.n, C, B, F));
  if (floats == 0) return DETAG_OK;
  return need_grad_scratch(ctx, floats, nullptr);
}

detag_status detag_gossip_accel(detag_ctx *ctx, void *Z_dev, int32_t K, double eta, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_state_ptr(ctx, Z_dev, "Z_dev")) return st;
  if (K < 0) return set_err(ctx, DETAG_EINVAL, "K must be >= 0");
  float e;
  if (detag_status st = resolve_eta(ctx, eta, &e)) return st;
  if (K == 0) return DETAG_OK;
  Chosen path;
  if (detag_status st = choose_path(ctx, &path)) return st;
  int rc = 0;
  switch (path) {
    case kFusedStructured:
      rc = launch_fused_structured(ctx->shape, ctx->W, 0, Z_dev, nullptr, nullptr, nullptr, 0.f, K, e, stream);
      break;
    case kFusedGeneric:
      rc = launch_fused_generic(ctx->shape, ctx->W, dev_csr(ctx), 0, Z_dev, nullptr, nullptr, nullptr, 0.f, K, e, stream);
      break;
    case kDense: {
      const uint16_t *frag = nullptr;
      if (detag_status st = dense_poly(ctx, K, e, &frag, stream)) return st;
      rc = launch_dense_phase(ctx->shape, 0, Z_dev, nullptr, nullptr, nullptr, 0.f, frag, stream);
      break;
    }
    case kPerRound: {
      WideState ws{ctx};
      if (detag_status st = ws.open(Z_dev, nullptr, stream)) return st;
      if (detag_status st = gossip_per_round_f32(ctx, ws.work[0], K, e, stream)) return st;
      return ws.close(stream);
    }
  }
  return rc ? hip_fail(ctx, "fused gossip", rc) : DETAG_OK;
}

detag_status detag_track(detag_ctx *ctx, void *Y_dev, const float *Gnew_dev, const float *Gold_dev, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_state_ptr(ctx, Y_dev, "Y_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, Gnew_dev, "Gnew_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, Gold_dev, "Gold_dev")) return st;
  const int rc = launch_track(ctx->shape, Y_dev, Gnew_dev, Gold_dev, stream);
  return rc ? hip_fail(ctx, "track", rc) : DETAG_OK;
}

detag_status detag_step(detag_ctx *ctx, void *X_dev, void *Y_dev, const float *Gnew_dev, const float *Gold_dev,
                        double alpha, int32_t K, double eta, int32_t variant, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_state_ptr(ctx, X_dev, "X_dev")) return st;
  if (detag_status st = check_state_ptr(ctx, Y_dev, "Y_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, Gnew_dev, "Gnew_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, Gold_dev, "Gold_dev")) return st;
  if (X_dev == Y_dev || static_cast<const void *>(Gnew_dev) == X_dev || static_cast<const void *>(Gnew_dev) == Y_dev ||
      static_cast<const void *>(Gold_dev) == X_dev || static_cast<const void *>(Gold_dev) == Y_dev)
    return set_err(ctx, DETAG_EINVAL, "X, Y and the gradient buffers must not overlap");
  if (K < 0) return set_err(ctx, DETAG_EINVAL, "K must be >= 0");
  if (!std::isfinite(alpha)) return set_err(ctx, DETAG_EINVAL, "alpha must be finite");
  if (variant != DETAG_VARIANT_ATC && variant != DETAG_VARIANT_ALG2)
    return set_err(ctx, DETAG_EINVAL, "unknown variant");
  float e;
  if (detag_status st = resolve_eta(ctx, eta, &e)) return st;
  const Shape &s = ctx->shape;
  const float a = float(alpha);
  if (K == 0) {  // M is the identity: both variants reduce to the two elementwise updates
    const int rc = launch_update_track(s, X_dev, Y_dev, Gnew_dev, Gold_dev, a, stream);
    return rc ? hip_fail(ctx, "update", rc) : DETAG_OK;
  }
  Chosen path;
  if (detag_status st = choose_path(ctx, &path)) return st;
  const int mode = variant == DETAG_VARIANT_ATC ? 1 : 2;
  if (path == kFusedStructured) {
    const int rc = launch_fused_structured(s, ctx->W, mode, X_dev, Y_dev, Gnew_dev, Gold_dev, a, K, e, stream);
    return rc ? hip_fail(ctx, "fused phase", rc) : DETAG_OK;
  }
  if (path == kFusedGeneric) {
    const int rc = launch_fused_generic(s, ctx->W, dev_csr(ctx), mode, X_dev, Y_dev, Gnew_dev, Gold_dev, a, K, e, stream);
    return rc ? hip_fail(ctx, "fused phase", rc) : DETAG_OK;
  }
  if (path == kDense) {
    const uint16_t *frag = nullptr;
    if (detag_status st = dense_poly(ctx, K, e, &frag, stream)) return st;
    const int rc = launch_dense_phase(s, mode, X_dev, Y_dev, Gnew_dev, Gold_dev, a, frag, stream);
    return rc ? hip_fail(ctx, "dense phase", rc) : DETAG_OK;
  }
  WideState ws{ctx};
  if (detag_status st = ws.open(X_dev, Y_dev, stream)) return st;
  const Shape sf = as_f32(s);
  if (variant == DETAG_VARIANT_ATC) {
    const int rc = launch_update_track(sf, ws.work[0], ws.work[1], Gnew_dev, Gold_dev, a, stream);
    if (rc) return hip_fail(ctx, "update", rc);
  }
  if (detag_status st = gossip_per_round_f32(ctx, ws.work[0], K, e, stream)) return st;
  if (detag_status st = gossip_per_round_f32(ctx, ws.work[1], K, e, stream)) return st;
  if (variant == DETAG_VARIANT_ALG2) {
    const int rc = launch_update_track(sf, ws.work[0], ws.work[1], Gnew_dev, Gold_dev, a, stream);
    if (rc) return hip_fail(ctx, "update", rc);
  }
  return ws.close(stream);
}

detag_status detag_dpsgd_step(detag_ctx *ctx, void *X_dev, const float *G_dev, double alpha, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_state_ptr(ctx, X_dev, "X_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, G_dev, "G_dev")) return st;
  if (!std::isfinite(alpha)) return set_err(ctx, DETAG_EINVAL, "alpha must be finite");
  if (static_cast<const void *>(G_dev) == X_dev) return set_err(ctx, DETAG_EINVAL, "X and G must not overlap");
  if (ctx->path != DETAG_PATH_PER_ROUND && fused_structured_available(ctx->W)) {  // one pass, 12 B per element
    const int rc = launch_fused_structured(ctx->shape, ctx->W, 3, X_dev, nullptr, G_dev, nullptr, float(alpha), 1, 0.f,
                                           stream);
    return rc ? hip_fail(ctx, "dpsgd", rc) : DETAG_OK;
  }
  if (round_stages_tile(ctx->shape)) {  // every column tile is read whole before it is written: in place, 12 B per element
    const int rc = launch_dpsgd(ctx->shape, dev_csr(ctx), X_dev, X_dev, G_dev, float(alpha), stream);
    return rc ? hip_fail(ctx, "dpsgd", rc) : DETAG_OK;
  }
  if (detag_status st = need_scratch(ctx, 0, 1, stream)) return st;
  int rc = launch_copy_state(ctx->shape, X_dev, ctx->scratch[0], stream);
  if (!rc) rc = launch_dpsgd(ctx->shape, dev_csr(ctx), ctx->scratch[0], X_dev, G_dev, float(alpha), stream);
  return rc ? hip_fail(ctx, "dpsgd", rc) : DETAG_OK;
}

detag_status detag_gossip_round(detag_ctx *ctx, const void *Zcur_dev, const void *Zprev_dev, void *Zout_dev, double eta,
                                void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_state_ptr(ctx, Zcur_dev, "Zcur_dev")) return st;
  if (detag_status st = check_state_ptr(ctx, Zprev_dev, "Zprev_dev")) return st;
  if (detag_status st = check_state_ptr(ctx, Zout_dev, "Zout_dev")) return st;
  if (Zout_dev == Zcur_dev) return set_err(ctx, DETAG_EINVAL, "Zout must not be Zcur: every neighbour reads Zcur");
  float e;
  if (detag_status st = resolve_eta(ctx, eta, &e)) return st;
  const int rc = round_launch(ctx, ctx->shape, Zcur_dev, Zprev_dev, Zout_dev, e, stream);
  return rc ? hip_fail(ctx, "gossip round", rc) : DETAG_OK;
}

detag_status detag_accumulate(detag_ctx *ctx, float *Gacc_dev, const float *g_dev, double scale, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_f32_ptr(ctx, Gacc_dev, "Gacc_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, g_dev, "g_dev")) return st;
  if (Gacc_dev == g_dev) return set_err(ctx, DETAG_EINVAL, "Gacc and g must not overlap");
  if (!std::isfinite(scale)) return set_err(ctx, DETAG_EINVAL, "scale must be finite");
  const int rc = launch_accumulate(ctx->shape, Gacc_dev, g_dev, float(scale), stream);
  return rc ? hip_fail(ctx, "accumulate", rc) : DETAG_OK;
}

detag_status detag_phase_end(detag_ctx *ctx, void *X_dev, void *Xt_dev, void *Y_dev, const float *Gk_dev,
                             float *Gkm1_dev, double alpha, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_state_ptr(ctx, X_dev, "X_dev")) return st;
  if (detag_status st = check_state_ptr(ctx, Xt_dev, "Xt_dev")) return st;
  if (detag_status st = check_state_ptr(ctx, Y_dev, "Y_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, Gk_dev, "Gk_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, Gkm1_dev, "Gkm1_dev")) return st;
  const void *p[5] = {X_dev, Xt_dev, Y_dev, Gk_dev, Gkm1_dev};
  for (int a = 0; a < 5; ++a)
    for (int b = a + 1; b < 5; ++b)
      if (p[a] == p[b] && !(a == 0 && b == 1))
        return set_err(ctx, DETAG_EINVAL, "the buffers must not overlap (X may be Xt)");
  if (!std::isfinite(alpha)) return set_err(ctx, DETAG_EINVAL, "alpha must be finite");
  const int rc = launch_phase_end(ctx->shape, X_dev, Xt_dev, Y_dev, Gk_dev, Gkm1_dev, float(alpha), stream);
  return rc ? hip_fail(ctx, "phase end", rc) : DETAG_OK;
}

namespace {
detag_status factors_create_impl(detag_ctx *ctx, int32_t root, detag_factors *f) {
  f->ctx = ctx;
  std::string err;
  if (!build_consensus_factors(ctx->W, root, f->host, err)) return set_err(ctx, DETAG_EINVAL, err);
  int64_t nnz = 0;
  for (auto &h : f->host) f->offs.push_back(nnz), nnz += int64_t(h.colidx.size());
  if (!build_factor_table(ctx->W.n, f->host, f->table)) f->table.clear();
  if (!ctx->has_device || f->host.empty()) return DETAG_OK;
  std::vector<int32_t> rp, ci;
  std::vector<float> va;
  for (auto &h : f->host) {
    rp.insert(rp.end(), h.rowptr.begin(), h.rowptr.end());
    ci.insert(ci.end(), h.colidx.begin(), h.colidx.end());
    for (double v : h.vals) va.push_back(float(v));
  }
  hipError_t e = hipMalloc(reinterpret_cast<void **>(&f->d_rowptr), rp.size() * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&f->d_colidx), ci.size() * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&f->d_vals), va.size() * sizeof(float));
  if (e == hipSuccess) e = hipMemcpy(f->d_rowptr, rp.data(), rp.size() * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(f->d_colidx, ci.data(), ci.size() * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(f->d_vals, va.data(), va.size() * sizeof(float), hipMemcpyHostToDevice);
  if (e == hipSuccess && !f->table.empty()) {
    const size_t bytes = f->table.size() * sizeof(uint32_t);
    e = hipMalloc(reinterpret_cast<void **>(&f->d_table), bytes);
    if (e == hipSuccess) e = hipMemcpy(f->d_table, f->table.data(), bytes, hipMemcpyHostToDevice);
  }
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return hip_fail(ctx, "factor upload", int(e));
  }
  return DETAG_OK;
}
}  // namespace

detag_status detag_factors_create(detag_ctx *ctx, int32_t root, detag_factors **out) {
  if (out) *out = nullptr;
  if (!ctx || !out) return set_err(ctx, DETAG_EINVAL, "ctx or out is NULL");
  auto *f = new (std::nothrow) detag_factors;
  if (!f) return set_err(ctx, DETAG_ENOMEM, "out of host memory");
  detag_status st;
  try {
    st = factors_create_impl(ctx, root, f);
  } catch (const std::bad_alloc &) {
    st = set_err(ctx, DETAG_ENOMEM, "out of host memory");
  }
  if (st != DETAG_OK) {
    detag_factors_destroy(f);
    return st;
  }
  *out = f;
  return DETAG_OK;
}

void detag_factors_destroy(detag_factors *f) {
  if (!f) return;
  if (f->d_rowptr || f->d_colidx || f->d_vals || f->d_table) {
    (void)hipDeviceSynchronize();
    (void)hipFree(f->d_rowptr);
    (void)hipFree(f->d_colidx);
    (void)hipFree(f->d_vals);
    (void)hipFree(f->d_table);
  }
  delete f;
}

detag_status detag_factors_count(const detag_factors *f, int32_t *R) {
  if (!f || !R) return DETAG_EINVAL;
  *R = int32_t(f->host.size());
  return DETAG_OK;
}

detag_status detag_factors_get_csr(const detag_factors *f, int32_t r, int64_t *nnz, const int32_t **rowptr,
                                   const int32_t **colidx, const double **vals) {
  if (!f) return DETAG_EINVAL;
  if (r < 0 || r >= int32_t(f->host.size())) return set_err(f->ctx, DETAG_EINVAL, "factor index out of range");
  const HostFactor &h = f->host[r];
  if (nnz) *nnz = int64_t(h.colidx.size());
  if (rowptr) *rowptr = h.rowptr.data();
  if (colidx) *colidx = h.colidx.data();
  if (vals) *vals = h.vals.data();
  return DETAG_OK;
}

detag_status detag_factors_get_program(const detag_factors *f, int64_t *batches, const uint32_t **words) {
  if (!f || !batches || !words) return DETAG_EINVAL;
  *batches = int64_t(f->table.size() / 32);
  *words = f->table.empty() ? nullptr : f->table.data();
  return DETAG_OK;
}

detag_status detag_factor_apply(detag_ctx *ctx, const detag_factors *f, int32_t r, const void *Zin_dev,
                                void *Zout_dev, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (!f || f->ctx != ctx) return set_err(ctx, DETAG_EINVAL, "the factors were not built for this context");
  if (r < 0 || r >= int32_t(f->host.size())) return set_err(ctx, DETAG_EINVAL, "factor index out of range");
  if (detag_status st = check_state_ptr(ctx, Zin_dev, "Zin_dev")) return st;
  if (detag_status st = check_state_ptr(ctx, Zout_dev, "Zout_dev")) return st;
  if (Zin_dev == Zout_dev) return set_err(ctx, DETAG_EINVAL, "Zout must not be Zin");
  DevCsr a;
  a.rowptr = f->d_rowptr + int64_t(r) * (ctx->W.n + 1);
  a.colidx = f->d_colidx + f->offs[r];
  a.vals = f->d_vals + f->offs[r];
  const int rc = launch_spmm(ctx->shape, a, Zin_dev, Zout_dev, stream);
  return rc ? hip_fail(ctx, "factor apply", rc) : DETAG_OK;
}

detag_status detag_average_consensus(detag_ctx *ctx, const detag_factors *f, void *Z_dev, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (!f || f->ctx != ctx) return set_err(ctx, DETAG_EINVAL, "the factors were not built for this context");
  if (detag_status st = check_state_ptr(ctx, Z_dev, "Z_dev")) return st;
  const int R = int(f->host.size());
  if (R == 0) return DETAG_OK;
  if (f->d_table && ctx->path != DETAG_PATH_PER_ROUND) {
    const int rc = launch_factor_sequence(ctx->shape, f->d_table, int(f->table.size()), Z_dev, stream);
    if (rc == 0) return DETAG_OK;
    if (rc > 0) return hip_fail(ctx, "factor sequence", rc);
    // rc < 0: does not fit the LDS of a block here; fall through to one launch per factor
  }
  // one launch per factor, between Z and a scratch matrix
  if (detag_status st = need_scratch(ctx, 0, 1, stream)) return st;
  void *cur = Z_dev, *other = ctx->scratch[0];
  for (int r = 0; r < R; ++r) {
    DevCsr a;
    a.rowptr = f->d_rowptr + int64_t(r) * (ctx->W.n + 1);
    a.colidx = f->d_colidx + f->offs[r];
    a.vals = f->d_vals + f->offs[r];
    if (int rc = launch_spmm(ctx->shape, a, cur, other, stream)) return hip_fail(ctx, "factor apply", rc);
    void *t = cur;
    cur = other, other = t;
  }
  if (cur != Z_dev)
    if (int rc = launch_copy_state(ctx->shape, cur, Z_dev, stream)) return hip_fail(ctx, "copy", rc);
  return DETAG_OK;
}

detag_status detag_defacto_update(detag_ctx *ctx, void *X_dev, void *Xt_dev, float *G_dev, double scale, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_state_ptr(ctx, X_dev, "X_dev")) return st;
  if (detag_status st = check_state_ptr(ctx, Xt_dev, "Xt_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, G_dev, "G_dev")) return st;
  if (static_cast<void *>(G_dev) == X_dev || static_cast<void *>(G_dev) == Xt_dev)
    return set_err(ctx, DETAG_EINVAL, "G must not overlap the models");
  if (!std::isfinite(scale)) return set_err(ctx, DETAG_EINVAL, "scale must be finite");
  const int rc = launch_defacto_update(ctx->shape, X_dev, Xt_dev, G_dev, float(scale), stream);
  return rc ? hip_fail(ctx, "defacto update", rc) : DETAG_OK;
}

detag_status detag_mean(detag_ctx *ctx, const void *X_dev, float *xbar_dev, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_state_ptr(ctx, X_dev, "X_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, xbar_dev, "xbar_dev")) return st;
  const int rc = launch_mean(ctx->shape, X_dev, xbar_dev, stream);
  return rc ? hip_fail(ctx, "mean", rc) : DETAG_OK;
}

detag_status detag_consensus_error(detag_ctx *ctx, const void *X_dev, double *sumsq_dev, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_state_ptr(ctx, X_dev, "X_dev")) return st;
  if (!sumsq_dev || misaligned(sumsq_dev, 8)) return set_err(ctx, DETAG_EINVAL, "sumsq_dev is NULL or misaligned");
  const int rc = launch_consensus_error(ctx->shape, X_dev, ctx->d_partials, sumsq_dev, stream);
  return rc ? hip_fail(ctx, "consensus error", rc) : DETAG_OK;
}

detag_status detag_consensus_error_static(detag_ctx *ctx, const void *X_dev, double *sumsq_dev, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_state_ptr(ctx, X_dev, "X_dev")) return st;
  if (!sumsq_dev || misaligned(sumsq_dev, 8)) return set_err(ctx, DETAG_EINVAL, "sumsq_dev is NULL or misaligned");
  if (consensus_partials_count(ctx->shape) > kStaticPartialsMax)
    return set_err(ctx, DETAG_EUNSUPPORTED,
                   "detag_consensus_error_static holds partial sums for d <= 16,777,216 columns; "
                   "use detag_consensus_error for wider matrices");
  int dev = -1;
  if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return hip_fail(ctx, "hipGetDevice", int(e));
  if (!static_partials(dev))
    if (int rc = static_partials_init(dev)) return hip_fail(ctx, "looking up the resident partial sums", rc);
  const int rc = launch_consensus_error(ctx->shape, X_dev, static_partials(dev), sumsq_dev, stream);
  return rc ? hip_fail(ctx, "consensus error", rc) : DETAG_OK;
}

detag_status detag_grad_quadratic_diag(detag_ctx *ctx, const void *X_dev, const float *h_dev, int32_t h_per_worker,
                                       const float *b_dev, const float *noise_dev, float sigma, uint64_t seed,
                                       uint32_t step, float *G_dev, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_state_ptr(ctx, X_dev, "X_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, h_dev, "h_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, b_dev, "b_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, G_dev, "G_dev")) return st;
  if (noise_dev && misaligned(noise_dev, 4)) return set_err(ctx, DETAG_EINVAL, "noise_dev is misaligned");
  if (static_cast<const void *>(G_dev) == X_dev) return set_err(ctx, DETAG_EINVAL, "G must not overlap X");
  if (!std::isfinite(sigma)) return set_err(ctx, DETAG_EINVAL, "sigma must be finite");
  const int rc = launch_grad_quadratic(ctx->shape, X_dev, h_dev, h_per_worker, b_dev, noise_dev, sigma, seed, step,
                                       G_dev, stream);
  return rc ? hip_fail(ctx, "quadratic gradient", rc) : DETAG_OK;
}

detag_status detag_step_quadratic(detag_ctx *ctx, void *X_dev, void *Y_dev, float *G_dev, const float *h_dev,
                                  int32_t h_per_worker, const float *b_dev, float sigma, uint64_t seed, uint32_t step, double alpha,
                                  int32_t K, double eta, int32_t variant, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (variant != DETAG_VARIANT_ATC && variant != DETAG_VARIANT_ALG2)
    return set_err(ctx, DETAG_EINVAL, "variant must be DETAG_VARIANT_ATC or DETAG_VARIANT_ALG2");
  if (detag_status st = check_state_ptr(ctx, X_dev, "X_dev")) return st;
  if (detag_status st = check_state_ptr(ctx, Y_dev, "Y_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, G_dev, "G_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, h_dev, "h_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, b_dev, "b_dev")) return st;
  if (X_dev == Y_dev || static_cast<void *>(G_dev) == X_dev || static_cast<void *>(G_dev) == Y_dev ||
      static_cast<const void *>(b_dev) == X_dev || static_cast<const void *>(b_dev) == Y_dev ||
      static_cast<const void *>(b_dev) == G_dev || static_cast<const void *>(h_dev) == X_dev ||
      static_cast<const void *>(h_dev) == Y_dev || static_cast<const void *>(h_dev) == G_dev)
    return set_err(ctx, DETAG_EINVAL, "X, Y, G, h and b must not overlap");
  if (!std::isfinite(alpha) || !std::isfinite(sigma)) return set_err(ctx, DETAG_EINVAL, "alpha and sigma must be finite");
  float e;
  if (detag_status st = resolve_eta(ctx, eta, &e)) return st;
  Chosen path = kPerRound;
  if (K >= 1)
    if (detag_status st = choose_path(ctx, &path)) return st;
  if (path != kFusedStructured && path != kFusedGeneric)
    return set_err(ctx, DETAG_EUNSUPPORTED,
                   "detag_step_quadratic needs K >= 1 and a context whose rounds run on chip (register-resident or "
                   "LDS-resident kernels, not the per-round or dense path)");
  int rc;
  if (path == kFusedStructured) {
    rc = launch_fused_quadratic(ctx->shape, ctx->W, variant == DETAG_VARIANT_ALG2, X_dev, Y_dev, G_dev, h_dev,
                                h_per_worker != 0, b_dev, float(alpha), K, e, sigma, seed, step, stream);
  } else {
    if (variant != DETAG_VARIANT_ATC)
      return set_err(ctx, DETAG_EUNSUPPORTED,
                     "Algorithm 2 as printed in one kernel needs the register-resident family (ring or torus on its "
                     "list); use detag_grad_quadratic_diag + detag_step");
    rc = launch_fused_generic_quadratic(ctx->shape, dev_csr(ctx), X_dev, Y_dev, G_dev, h_dev, h_per_worker != 0, b_dev,
                                        float(alpha), K, e, sigma, seed, step, stream);
  }
  return rc ? hip_fail(ctx, "fused gradient + phase", rc) : DETAG_OK;
}

detag_status detag_grad_lstsq(detag_ctx *ctx, const void *X_dev, const float *A_dev, const float *b_dev, int32_t m,
                              float *G_dev, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (detag_status st = check_state_ptr(ctx, X_dev, "X_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, A_dev, "A_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, b_dev, "b_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, G_dev, "G_dev")) return st;
  if (m < 1) return set_err(ctx, DETAG_EINVAL, "m must be >= 1");
  if (detag_status st = need_grad_scratch(ctx, int64_t(ctx->shape.n) * m, stream)) return st;
  const int rc = launch_grad_lstsq(ctx->shape, X_dev, A_dev, b_dev, m, ctx->d_resid, G_dev, stream);
  return rc ? hip_fail(ctx, "least-squares gradient", rc) : DETAG_OK;
}

detag_status detag_grad_softmax_bf16(detag_ctx *ctx, const void *X_dev, const uint16_t *feat_dev,
                                     const int32_t *labels_dev, const int32_t *batch_dev, int32_t S, int32_t F,
                                     int32_t C, int32_t B, float *G_dev, float *loss_dev, void *stream) {
  if (detag_status st = need_device(ctx)) return st;
  if (ctx->shape.bf16) return set_err(ctx, DETAG_EUNSUPPORTED, "softmax gradient needs fp32 state");
  if (detag_status st = check_state_ptr(ctx, X_dev, "X_dev")) return st;
  if (detag_status st = check_f32_ptr(ctx, G_dev, "G_dev")) return st;
  if (!feat_dev || !labels_dev || !batch_dev) return set_err(ctx, DETAG_EINVAL, "a data pointer is NULL");
  if (misaligned(feat_dev, 16) || misaligned(labels_dev, 4) || misaligned(batch_dev, 4) ||
      (loss_dev && misaligned(loss_dev, 4)))
    return set_err(ctx, DETAG_EINVAL, "a data pointer is misaligned (features need 16 bytes)");
  if (C < 2 || C > 10 || F < 32 || F % 32 || B < 32 || B % 32 || B > 256 || S < 1)
    return set_err(ctx, DETAG_EUNSUPPORTED, "softmax gradient limits: 2 <= C <= 10, F % 32 == 0, B % 32 == 0, B <= 256");
  if (int64_t(C) * F + C != ctx->shape.d)
    return set_err(ctx, DETAG_EINVAL, "d must equal C*F + C");
  if (detag_status st = need_grad_scratch(ctx, softmax_scratch_floats(ctx->shape.n, C, B, F), stream)) return st;
  const int rc = launch_grad_softmax(ctx->shape, X_dev, feat_dev, labels_dev, batch_dev, S, F, C, B, ctx->d_resid,
                                     G_dev, loss_dev, stream);
  return rc ? hip_fail(ctx, "softmax gradient", rc) : DETAG_OK;
}

const char *detag_last_error(const detag_ctx *ctx) { return ctx ? ctx->err.c_str() : g_create_err.c_str(); }

const char *detag_version(void) { return "detag-gfx950 0.1"; }

}  // extern "C"
