// Internal declarations shared by the host code and the kernel launchers.
// Nothing here is part of the C ABI (see include/detag.h).
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "detag.h"

namespace detag {

// Structured neighbour patterns the register-resident kernels are compiled for.
enum Structure : int { kGeneric = 0, kRing = 1, kTorus = 2 };

// The gossip matrix on the host.  Row i of the CSR lists (j, W_ji), j ascending,
// self included: exactly the terms of worker i's gossip sum.
struct HostW {
  int n = 0;
  std::vector<int32_t> rowptr, colidx;
  std::vector<double> vals;
  bool symmetric = false;
  double lambda2 = 0, lambdan = 0, lambda = 0, eta = 0;  // NaN when not symmetric
  Structure structure = kGeneric;
  int trows = 0, tcols = 0;       // torus shape
  double w_self = 0, w_nb = 0;    // structured patterns: one self weight, one neighbour weight
  int max_row_nnz = 0;
};

// Builds, validates and analyses W.  On failure returns the status and fills err.
detag_status build_gossip_matrix(const detag_topology *topo, int n, HostW &W, std::string &err);

// One factor of the average-consensus product, as a CSR whose row i lists (j, A_ij), j ascending:
// applying it is x_i <- sum_j A_ij x_j (in Algorithm 1's notation A_ij = [W_r]_ji).
struct HostFactor {
  std::vector<int32_t> rowptr, colidx;
  std::vector<double> vals;
};
// Spanning-tree (gather, then propagate) factors on the undirected support of W, rooted at `root`.
bool build_consensus_factors(const HostW &W, int root, std::vector<HostFactor> &out, std::string &err);

// Device table of a factor sequence for the on-chip kernel: batches of four 4-word operations (header, two packed
// 16-bit LDS byte offsets, two fp32 weights) covering the non-identity rows of every factor in an order the kernel
// may execute batch by batch.  false if n > 256, a factor row has more than 8 terms, or the rows a step changes
// read each other in a cycle.
bool build_factor_table(int n, const std::vector<HostFactor> &factors, std::vector<uint32_t> &table);

// Eigenvalues (ascending) of a dense symmetric matrix, cyclic Jacobi. a is n*n row-major, destroyed.
void symmetric_eigenvalues(std::vector<double> &a, int n, std::vector<double> &ev);

// ---------------------------------------------------------------------------
// Kernel launchers.  All pointers are device pointers; stream is a hipStream_t.
// Each returns a hipError_t value as int (0 = success).
// ---------------------------------------------------------------------------
struct DevCsr {
  const int32_t *rowptr = nullptr;  // n+1
  const int32_t *colidx = nullptr;  // nnz
  const float *vals = nullptr;      // nnz, fp32 copies of W_ji
  // the same matrix for the on-chip kernel for arbitrary W: one packed record per row (see EllHost)
  const uint32_t *ell_table = nullptr;
  int ell_deg = 0;
  bool ell_uniform = false;
};

// Neighbour table of the on-chip kernel for arbitrary W (256 row slots, wavefront-major: row i sits at slot
// (i % 16) * 16 + i / 16).  Per slot: deg/2 words of packed 16-bit LDS byte offsets of the neighbours' rows, then
// the off-diagonal weights as fp32 bit patterns (one word if every row has equal off-diagonal weights, else deg
// words).  Missing neighbours point at the row itself: the kernel works with differences z_j - z_i, so they
// contribute nothing.
struct EllHost {
  int deg = 0;            // table width: 2, 4 or 8
  bool uniform = false;   // each row's off-diagonal weights are all equal
  std::vector<uint32_t> table;
};
// false if W has more than 256 rows or a row with more than 8 off-diagonal terms.
bool build_ell(const HostW &W, EllHost &out);

struct Shape {
  int n;
  int64_t d, ld;
  bool bf16;  // storage of X/Y
};

// Z <- A_{R-1} ... A_0 Z on chip, in place (table from build_factor_table).  -1 if n rows of 64 columns do not
// fit a block's LDS on this device.
int launch_factor_sequence(const Shape &s, const uint32_t *table, int table_words, void *Z, void *stream);
// The matrix polynomial of K rounds of Algorithm 3, P = p_K(W^T), as bf16 terms in the operand order of
// dense_phase_kernel (`terms` = dense_poly_terms(state type), dense_poly_words(terms) 16-bit words).  false if n > 256.
void gossip_polynomial(const HostW &W, int K, double eta, std::vector<double> &P);  // n x n, row-major, fp64
int dense_poly_terms(bool bf16_state);
size_t dense_poly_words(int terms);
bool build_dense_poly(const HostW &W, int K, double eta, int terms, std::vector<uint16_t> &frag);
// One phase with P: mode 0: X <- P X.  mode 1: X <- P (X - alpha*Y), Y <- P (Y + Gn - Go).
// mode 2: X <- P X - alpha * P Y (evaluated as P (X - alpha*Y)), Y <- P Y + Gn - Go.  n <= 256.
int launch_dense_phase(const Shape &s, int mode, void *X, void *Y, const float *Gn, const float *Go, float alpha,
                       const uint16_t *frag, void *stream);
// out = A cur for a CSR matrix A whose rows need not sum to one (row i lists (j, A_ij)); out != cur.
int launch_spmm(const Shape &s, const DevCsr &a, const void *cur, void *out, void *stream);
// X = Xt - scale*G; Xt = X; G = 0   (X may be Xt)
int launch_defacto_update(const Shape &s, void *X, void *Xt, float *G, float scale, void *stream);
// One round of Algorithm 3, out = (1+eta) * (W^T cur) - eta * prev.  out may alias prev; out != cur.
int launch_gossip_round(const Shape &s, const DevCsr &w, const void *cur, const void *prev, void *out, float eta,
                        void *stream);
// Y += Gnew - Gold
int launch_track(const Shape &s, void *Y, const float *Gn, const float *Go, void *stream);
// X -= alpha*Y (old Y); Y += Gnew - Gold   (one pass)
int launch_update_track(const Shape &s, void *X, void *Y, const float *Gn, const float *Go, float alpha,
                        void *stream);
// X = c_mix * (W^T Xin) - alpha*G  (D-PSGD); Xin != X
bool round_stages_tile(const Shape &s);
int launch_structured_round(const Shape &s, const HostW &W, const void *cur, const void *prev, void *out, float eta,
                            void *stream);
int launch_dpsgd(const Shape &s, const DevCsr &w, const void *Xin, void *X, const float *G, float alpha,
                 void *stream);
int launch_copy_state(const Shape &s, const void *src, void *dst, void *stream);
// Gacc += scale * g (fp32 n x ld)
int launch_accumulate(const Shape &s, float *Gacc, const float *g, float scale, void *stream);
// X = Xt - alpha*Y; Y += Gk - Gkm1; Xt = X; Gkm1 = 0   (X may be Xt)
int launch_phase_end(const Shape &s, void *X, void *Xt, void *Y, const float *Gk, float *Gkm1, float alpha,
                     void *stream);
// n x ld matrices: bf16 -> fp32 (exact) and fp32 -> bf16 (round to nearest even)
int launch_widen(const Shape &s, const void *src_bf16, float *dst, void *stream);
int launch_narrow(const Shape &s, const float *src, void *dst_bf16, void *stream);

// Fused K-round kernels.  mode: 0 = gossip only on X (Y, Gn, Go unused), 1 = ATC phase, 2 = ALG2 phase.
// Returns -1 if no kernel exists for this (structure, n).
bool fused_structured_available(const HostW &W);
int launch_fused_structured(const Shape &s, const HostW &W, int mode, void *X, void *Y, const float *Gn,
                            const float *Go, float alpha, int K, float eta, void *stream);
// Gradient query of the diagonal quadratic + ATC phase in one kernel; G holds g(k-1) on entry, g(k) on exit.
int launch_fused_quadratic(const Shape &s, const HostW &W, bool alg2, void *X, void *Y, float *G, const float *h,
                           bool h_per_worker, const float *b, float alpha, int K, float eta, float sigma, uint64_t seed,
                           uint32_t step, void *stream);
bool fused_generic_available(const HostW &W, const Shape &s);
int launch_fused_generic_quadratic(const Shape &s, const DevCsr &w, void *X, void *Y, float *G, const float *h,
                                   bool h_per_worker, const float *b, float alpha, int K, float eta, float sigma,
                                   uint64_t seed, uint32_t step, void *stream);
int launch_fused_generic(const Shape &s, const HostW &W, const DevCsr &w, int mode, void *X, void *Y,
                         const float *Gn, const float *Go, float alpha, int K, float eta, void *stream);

// Diagnostics
int launch_mean(const Shape &s, const void *X, float *xbar, void *stream);
int64_t consensus_partials_count(const Shape &s);
int launch_consensus_error(const Shape &s, const void *X, double *partials, double *out, void *stream);
// The library-resident partial-sum array of detag_consensus_error_static: kStaticPartialsMax doubles per GPU.
// static_partials_init looks its address up on `device` (which must be current), once; static_partials returns
// that address, or nullptr before a successful init.
constexpr int64_t kStaticPartialsMax = 65536;  // 512 KiB; one slot per 256 columns: d <= 16,777,216
int static_partials_init(int device);
double *static_partials(int device);

// Gradients
int launch_grad_quadratic(const Shape &s, const void *X, const float *h, int h_per_worker, const float *b,
                          const float *noise, float sigma, uint64_t seed, uint32_t step, float *G,
                          void *stream);
int launch_grad_lstsq(const Shape &s, const void *X, const float *A, const float *b, int m, float *resid,
                      float *G, void *stream);
int64_t softmax_scratch_floats(int n, int C, int B, int F);
int launch_grad_softmax(const Shape &s, const void *X, const uint16_t *feat, const int32_t *labels,
                        const int32_t *batch, int S, int F, int C, int B, float *scratch, float *G, float *loss,
                        void *stream);

}  // namespace detag
