/*
 * detag.h — C ABI of the DeTAG hot path on one AMD MI355X (gfx950).
 *
 * The library simulates all n workers of a decentralized data-parallel run on
 * one GPU.  Every state matrix (models X, gradient trackers Y, gradients G) is
 * n x ld row-major in device memory: row i is worker i, the d parameters of a
 * worker are contiguous, ld >= d is the row pitch in elements, and the columns
 * [d, ld) are padding the library neither reads nor writes.
 *
 * Paper: Lu & De Sa, "Optimal Complexity in Decentralized Training"
 * (arXiv 2006.08085).  Each entry point cites the passage that defines it.
 *
 * Conventions shared by all entry points
 *   - Pointers named *_dev are DEVICE pointers owned by the caller; the
 *     library never frees or keeps them after the call's work is enqueued.
 *     All other pointers are HOST pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All device work is enqueued on it; no entry point synchronises the
 *     host unless its comment says so, with one exception: memory the context
 *     owns (per-round scratch, gradient scratch, the dense path's polynomial)
 *     is allocated by the first call that needs it, unless detag_reserve_*
 *     did so before.  Results written to *_dev outputs are valid once the
 *     stream reaches them.
 *   - Enumerated arguments cross the ABI as int32_t (the enum types below name
 *     their values): a value outside the enumeration is an ordinary bad
 *     argument, answered with DETAG_EINVAL.
 *   - Calls return a detag_status; nothing throws or aborts across the ABI.
 *     detag_last_error() gives the text of the last failure.
 *   - Calls on one context come from one host thread at a time.  Work of two
 *     calls may run concurrently on two streams only if they use disjoint
 *     context-owned scratch: detag_gossip_round, detag_accumulate,
 *     detag_phase_end, detag_track, detag_grad_quadratic_diag and the on-chip
 *     paths of detag_gossip_accel / detag_step / detag_dpsgd_step use none;
 *     the per-round paths share one scratch area, the least-squares and
 *     softmax gradients another, the two diagnostics a third.
 *     State matrices passed to one call must not overlap unless the comment
 *     allows it.
 */
#ifndef DETAG_H
#define DETAG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct detag_ctx detag_ctx; /* opaque; owned by the library */

typedef enum {
  DETAG_OK = 0,
  DETAG_EINVAL = 1,                /* bad argument (null, size, range, alignment) */
  DETAG_ENOT_DOUBLY_STOCHASTIC = 2,/* a row or column of W does not sum to 1, or a weight is negative */
  DETAG_EDISCONNECTED = 3,         /* the support graph of W is not connected (lambda = 1) */
  DETAG_EUNSUPPORTED = 4,          /* valid request the library has no kernel for */
  DETAG_ENOMEM = 5,                /* host or device allocation failed */
  DETAG_EHIP = 6                   /* HIP runtime error, or no GPU present */
} detag_status;

/* Storage type of X and Y.  Gradients are always fp32; arithmetic is fp32. */
typedef enum { DETAG_F32 = 0, DETAG_BF16 = 1 } detag_dtype;

typedef enum {
  DETAG_TOPO_RING = 0,           /* cycle over n workers (n = 2: one edge; n = 1: no edge) */
  DETAG_TOPO_TORUS2D = 1,        /* rows x cols grid with wrap-around, n = rows*cols */
  DETAG_TOPO_RANDOM_REGULAR = 2, /* seeded random `degree`-regular graph (degree even) */
  DETAG_TOPO_EDGES = 3,          /* caller's undirected edge list */
  DETAG_TOPO_CSR = 4             /* caller's complete W in CSR, see below */
} detag_topo_kind;

typedef enum {
  DETAG_W_UNIFORM = 0,   /* 1/(deg+1) on every edge and self-loop; regular graphs only */
  DETAG_W_METROPOLIS = 1 /* 1/(1+max(deg_i,deg_j)) per edge, remainder on the diagonal */
} detag_weight_kind;

/*
 * The gossip matrix W of the paper's class W_n ("Protocol Layer": doubly
 * stochastic, W_ij != 0 only on edges of the graph or the diagonal).
 *   kind RING / TORUS2D / RANDOM_REGULAR / EDGES: the library builds W from
 *     the graph with `weights`.
 *   kind CSR: the caller gives W itself.  Row i of the CSR lists the pairs
 *     (j, W_ji) — the terms of the gossip sum of worker i, which reads
 *     column i of W; the self term must be listed.  `weights` is ignored.
 *   kappa: slack matrix W_kappa = kappa*W + (1-kappa)*I ("Experiments",
 *     second experiment); 1.0 leaves W unchanged.  Must be in (0, 1].
 * All arrays are host memory, read during detag_create only.
 */
typedef struct {
  int32_t kind;          /* detag_topo_kind */
  int32_t weights;       /* detag_weight_kind */
  int32_t rows, cols;    /* TORUS2D only */
  int32_t degree;        /* RANDOM_REGULAR only */
  uint64_t seed;         /* RANDOM_REGULAR only */
  double kappa;
  int64_t n_edges;       /* EDGES: number of pairs in `edges` */
  const int32_t *edges;  /* EDGES: 2*n_edges vertex ids, pairs (a,b), a != b, no repeats */
  const int32_t *rowptr; /* CSR: n+1 offsets */
  const int32_t *colidx; /* CSR: nnz worker ids j */
  const double *vals;    /* CSR: nnz weights W_ji */
} detag_topology;

/* Which form of the phase update detag_step applies. */
typedef enum {
  DETAG_VARIANT_ATC = 0, /* matrix form in the proof of Theorem 3: Y+ = M(Y+Gnew-Gold), X+ = M(X-alpha*Y) */
  DETAG_VARIANT_ALG2 = 1 /* Algorithm 2 as printed: gossip first, then x = x~ - alpha*y, y = y + g(k) - g(k-1) */
} detag_variant;

/* Which kernels run the accelerated gossip; AUTO picks the fastest that applies. */
typedef enum {
  DETAG_PATH_AUTO = 0,
  DETAG_PATH_PER_ROUND = 1, /* one launch per gossip round, state streamed through HBM every round */
  DETAG_PATH_FUSED = 2,     /* all K rounds on chip, one pass over the state; EUNSUPPORTED if n does not fit */
  /* The K rounds as one product with the matrix polynomial of Algorithm 3, P = p_K(W^T),
   * p_{k+1}(M) = (1+eta) M p_k(M) - eta p_{k-1}(M), p_0 = p_{-1} = I, on the matrix cores (n <= 256, else
   * EUNSUPPORTED): same result up to rounding, cost independent of K and of the graph's degree.  Applies to
   * detag_gossip_accel and detag_step; the first call with a new (K, eta) evaluates P on the host and uploads
   * it (a blocking copy; the context keeps the last four).  AUTO never picks it. */
  DETAG_PATH_DENSE = 3
} detag_path;

/*
 * Build W, check it, compute its spectrum and eta, and upload the neighbour
 * lists.  Host work only, plus one small synchronous upload.
 *   n  workers (>= 1), d parameters per worker (>= 1), ld row pitch (>= d).
 *   state: storage type of X and Y for every later call on this context.
 * Rejects: n < 1, d < 1, ld < d, kappa outside (0,1], a malformed graph or
 * CSR (EINVAL); row/column sums off 1 by more than 1e-9 or negative weights
 * (ENOT_DOUBLY_STOCHASTIC); a disconnected support graph (EDISCONNECTED).
 * lambda = max(|lambda_2|, |lambda_n|) ("Protocol Layer") and
 * eta = (1-sqrt(1-lambda^2))/(1+sqrt(1-lambda^2)) (Algorithm 3) are computed
 * when W is symmetric; for an asymmetric W they are NaN and every call must
 * pass eta explicitly.  n = 1: W = [1], lambda = eta = 0.
 * Without a GPU the context is still created (spectrum and CSR can be
 * queried); every device entry point then returns DETAG_EHIP.
 * On failure *out is NULL and detag_last_error(NULL) has the reason.
 */
detag_status detag_create(const detag_topology *topo, int32_t n, int64_t d, int64_t ld,
                          int32_t state /* detag_dtype */, detag_ctx **out);

/* Frees the context and its device scratch.  Synchronises the device. NULL is ignored. */
void detag_destroy(detag_ctx *ctx);

/* lambda_2, lambda_n, lambda, eta of the context's W (host doubles; any may be NULL). */
detag_status detag_get_spectrum(const detag_ctx *ctx, double *lambda2, double *lambdan,
                                double *lambda, double *eta);

/*
 * Phase length suggested by Theorem 3 for the context's W:
 *   R = max(log(n)/2, log(outer_ratio)/2) / sqrt(1 - lambda), rounded up, at least 1,
 * with outer_ratio = varsigma_0^2 T / (Delta L) in the theorem's notation; pass a
 * value <= 0 to leave that term out (R then depends on n and lambda only).
 * DETAG_EINVAL if W has no stored lambda (asymmetric W) or R does not fit an int32.
 */
detag_status detag_get_phase_length(const detag_ctx *ctx, double outer_ratio, int32_t *R);

/* Host views of W as stored (row i = pairs (j, W_ji), self included, j ascending).
 * The arrays belong to the context and live until detag_destroy. */
detag_status detag_get_csr(const detag_ctx *ctx, int32_t *n, int64_t *nnz, const int32_t **rowptr,
                           const int32_t **colidx, const double **vals);

/* Select the gossip kernels (default AUTO).  FUSED is refused with EUNSUPPORTED
 * if the context's n has no on-chip kernel. */
detag_status detag_set_path(detag_ctx *ctx, int32_t path /* detag_path */);

/*
 * Which kernel family detag_gossip_accel and detag_step (K >= 1) run on this
 * context with its current path: it depends on the topology and on n, and the
 * families differ in cost by integer factors, so a caller sizing a run should
 * look.  Measured on MI355X, fp32 state unless noted:
 *   DETAG_KERNEL_REGISTER_TILE  ring with n in {4, 8, 12, 16, 24, 32, 48,
 *     64}, torus 4x4, 4x8, 8x8 (built from DETAG_TOPO_RING / DETAG_TOPO_TORUS2D with uniform
 *     weights and any kappa).  All n rows of a column in registers, K rounds
 *     on chip: 24 B per element and phase whatever K is, 0.66 of HBM peak at
 *     n = 64, d = 11.2 M.  Only this family serves detag_step_quadratic with
 *     DETAG_VARIANT_ALG2 and the one-pass detag_dpsgd_step.
 *   DETAG_KERNEL_LDS_TILE  any other W with n <= 256 and at most 8 neighbours
 *     per worker, including rings and tori off the list above.  Same HBM
 *     bytes, but the rounds run at LDS bandwidth: per phase about
 *     0.9 ms + K * 0.16 ms at n = 256, d = 1 M (bf16 state), where HBM alone
 *     would take 0.6 ms: 4 to 5 times the register family's time per byte
 *     at K = 16, on par with it at K = 1.  A block has 16, 32, 64, 128 or
 *     256 row slots (the smallest count that holds n), and its time goes with
 *     the slots: a 1 GiB fp32 matrix takes 1.0-1.2 ms per 8-round gossip for
 *     n = 24 ... 256, 1.7 ms for n = 12, 2.8 ms for n = 7.
 *   DETAG_KERNEL_PER_ROUND  everything else (n > 256, a worker with more than 8
 *     neighbours), or DETAG_PATH_PER_ROUND: one launch per round, 12 B per
 *     element and round (24 + 8*(3K-1) B per element and phase: 208 B at K = 8,
 *     nine times the on-chip families).
 *   DETAG_KERNEL_DENSE  only after detag_set_path(DETAG_PATH_DENSE).
 */
typedef enum {
  DETAG_KERNEL_PER_ROUND = 0,
  DETAG_KERNEL_REGISTER_TILE = 1,
  DETAG_KERNEL_LDS_TILE = 2,
  DETAG_KERNEL_DENSE = 3
} detag_kernel;
detag_status detag_get_kernel(const detag_ctx *ctx, int32_t *kernel /* detag_kernel */);

/* 1 if the fused (all K rounds on chip) kernels exist for this context, else 0. */
int32_t detag_has_fused(const detag_ctx *ctx);

/*
 * The matrix of K rounds of Algorithm 3 with momentum eta (eta < 0: the context's): AG_K(Z) = P Z with
 * P = p_K(W^T), p_0 = p_{-1} = I, p_{k+1}(M) = (1+eta) M p_k(M) - eta p_{k-1}(M).  Host work only, fp64;
 * P_out: n*n doubles, row-major, caller-owned.  For a symmetric W its singular values are |p_K(mu)| over W's
 * eigenvalues mu, so it gives the exact contraction of the K rounds; DETAG_PATH_DENSE multiplies by it.
 */
detag_status detag_get_gossip_polynomial(const detag_ctx *ctx, int32_t K, double eta, double *P_out);

/*
 * Memory the library owns is allocated on first use: the per-round path's
 * scratch matrices, the dense path's uploaded polynomial for a (K, eta), the
 * gradient scratch.  Such a first use allocates, and for the polynomial also
 * blocks the host.  The two calls below do that work up front, so that every
 * later call only enqueues kernels; they are what a caller needs before it
 * records calls into a HIP graph.  While `stream` is being captured, an entry
 * point that would still have to allocate returns DETAG_EINVAL and enqueues
 * nothing.
 *
 * detag_reserve_gossip: path = DETAG_PATH_PER_ROUND reserves the scratch of
 *   detag_gossip_accel / detag_step / detag_dpsgd_step / detag_average_consensus
 *   on that path (K and eta are ignored); path = DETAG_PATH_DENSE evaluates
 *   and uploads the polynomial for (K, eta) (eta < 0: the context's eta) into
 *   the context's cache of four.
 * detag_reserve_gradient: m > 0 reserves for detag_grad_lstsq with that m;
 *   F, C, B > 0 for detag_grad_softmax_bf16 with those sizes; zeros skip.
 * Both may allocate and block; call them outside any capture.
 */
detag_status detag_reserve_gossip(detag_ctx *ctx, int32_t path /* detag_path */, int32_t K, double eta);
detag_status detag_reserve_gradient(detag_ctx *ctx, int32_t m, int32_t F, int32_t C, int32_t B);

/*
 * Accelerated gossip, Algorithm 3, for all workers at once, in place:
 *   z_{-1} = z_0;  z_{r+1} = (1+eta) * sum_{j in N_i + i} z_{r,j} W_ji - eta * z_{r-1,i},  r = 0..K-1.
 * Z_dev: n x ld matrix of the context's state type; holds z_K on return.
 * K >= 0 (K = 0 is a no-op).  eta in [0,1), or negative to use the context's eta.
 * The per-round path allocates its scratch (two n x ld matrices) on first use.
 */
detag_status detag_gossip_accel(detag_ctx *ctx, void *Z_dev, int32_t K, double eta, void *stream);

/*
 * Tracker update of Algorithm 2: Y <- Y + Gnew - Gold, in place on Y.
 * Y_dev: state type; Gnew_dev, Gold_dev: fp32, n x ld.
 */
detag_status detag_track(detag_ctx *ctx, void *Y_dev, const float *Gnew_dev, const float *Gold_dev,
                         void *stream);

/*
 * One DeTAG phase of length K (Algorithm 2 with R = K, all workers), in place
 * on X and Y.  Gradients are inputs: Gnew = this phase's gradient buffer g(k),
 * Gold = the previous one g(k-1); the caller swaps them afterwards.
 *   ATC : X+ = M(X - alpha*Y);  Y+ = M(Y + Gnew - Gold)       (proof of Theorem 3)
 *   ALG2: X+ = M(X) - alpha*M(Y);  Y+ = M(Y) + Gnew - Gold    (Algorithm 2 as printed)
 * with M the K-step accelerated gossip above.  eta as in detag_gossip_accel.
 * X_dev, Y_dev: state type; Gnew_dev, Gold_dev: fp32.  The four must not overlap.
 */
detag_status detag_step(detag_ctx *ctx, void *X_dev, void *Y_dev, const float *Gnew_dev,
                        const float *Gold_dev, double alpha, int32_t K, double eta,
                        int32_t variant /* detag_variant */, void *stream);

/*
 * D-PSGD, the baseline of the "Experiments" section: X <- W^T X - alpha*G,
 * in place on X (one plain gossip step of the models, then the local step).
 */
detag_status detag_dpsgd_step(detag_ctx *ctx, void *X_dev, const float *G_dev, double alpha, void *stream);

/*
 * Algorithm 2 at the granularity it is printed in: one iteration = one step of
 * accelerated gossip on the model replica and on the tracker (these calls, on
 * a communication stream) while gradient queries at the phase-start model
 * accumulate in the gradient buffer (detag_accumulate, on another stream); the
 * last iteration of a phase ends with detag_phase_end.
 *
 * detag_gossip_round: one step of Algorithm 3,
 *   Zout = (1+eta) * W^T Zcur - eta * Zprev.
 * Zprev == Zcur for the first step of a phase (z_{-1} = z_0).  Zout may be the
 * same buffer as Zprev (each output element reads only its own previous
 * value); it must not be Zcur.  All three: n x ld, state type.  The caller
 * rotates the buffers.  eta as in detag_gossip_accel.  With bf16 state every
 * call rounds its output (the fused entry points round once per phase).
 * Every row is read once (12 B per element with fp32 state) on ring and torus
 * contexts of the register-resident family and, for any other W with
 * n <= 256, on matrices of 128 MiB and more; smaller ones and n > 256 read a
 * row once per neighbour, mostly from the caches.
 */
detag_status detag_gossip_round(detag_ctx *ctx, const void *Zcur_dev, const void *Zprev_dev, void *Zout_dev,
                                double eta, void *stream);

/* Gradient buffer of Algorithm 2: Gacc += scale * g  (both fp32 n x ld; Gacc != g). */
detag_status detag_accumulate(detag_ctx *ctx, float *Gacc_dev, const float *g_dev, double scale, void *stream);

/*
 * End of a phase of Algorithm 2 (its last four lines), with Xt the gossiped model
 * replica and Y the gossiped tracker:
 *   X <- Xt - alpha*Y;   Y <- Y + Gk - Gkm1;   Xt <- X;   Gkm1 <- 0.
 * Gk holds the phase's accumulated gradients g(k), Gkm1 those of the phase
 * before; on return Gkm1 is cleared, ready to be the next phase's accumulation
 * buffer once the caller has swapped the two pointers (g(k-1) <- g(k), g(k) <- 0).
 * X_dev, Xt_dev, Y_dev: state type; Gk_dev, Gkm1_dev: fp32.  X_dev may equal Xt_dev
 * (no separate replica); otherwise the five must not overlap.
 */
detag_status detag_phase_end(detag_ctx *ctx, void *X_dev, void *Xt_dev, void *Y_dev, const float *Gk_dev,
                             float *Gkm1_dev, double alpha, void *stream);

/*
 * DeFacto (Algorithm 1) and the exact average consensus it communicates with
 * (Lemma 1): a sequence of R matrices with the sparsity of the context's graph
 * whose product is 11^T/n.  The factors are the spanning-tree construction of
 * the paper's supplementary material (gather to a root level by level, then
 * propagate back), built on the host at creation: R = 2 * (depth of the
 * breadth-first tree from `root`), between D and 2D for a graph of diameter D.
 * Factor r is stored as a CSR whose row i lists (j, A_ij), j ascending, and is
 * applied as  z_i <- sum_j A_ij z_j,  i.e. A_ij = [W_r]_ji in Algorithm 1's
 * notation; applying r = 0, ..., R-1 in order leaves every worker with the mean.
 */
typedef struct detag_factors detag_factors;

/* Builds the factors for the graph of ctx's W (undirected support of its off-diagonal entries).
 * The factors belong to ctx's device and must be destroyed before ctx.  DETAG_EINVAL for a bad root. */
detag_status detag_factors_create(detag_ctx *ctx, int32_t root, detag_factors **out);
void detag_factors_destroy(detag_factors *f);
/* Number of factors R. */
detag_status detag_factors_count(const detag_factors *f, int32_t *R);
/* Host view of factor r (arrays live until detag_factors_destroy). */
detag_status detag_factors_get_csr(const detag_factors *f, int32_t r, int64_t *nnz, const int32_t **rowptr,
                                   const int32_t **colidx, const double **vals);
/* Zout = A_r Zin: the communication step of Algorithm 1 with the r-th factor.  n x ld, state type; Zout != Zin. */
detag_status detag_factor_apply(detag_ctx *ctx, const detag_factors *f, int32_t r, const void *Zin_dev,
                                void *Zout_dev, void *stream);
/*
 * All R factors in order, in place: Z <- A_{R-1} ... A_0 Z, after which every worker's row is the column mean
 * (the R communication iterations of a round of Algorithm 1 as one call).  With up to 256 workers and at most
 * 8 terms per factor row the whole sequence runs on chip and Z crosses memory once; otherwise (or with
 * DETAG_PATH_PER_ROUND) it is one launch per factor through a context-owned scratch matrix.
 */
detag_status detag_average_consensus(detag_ctx *ctx, const detag_factors *f, void *Z_dev, void *stream);
/*
 * Host view of what the on-chip form of detag_average_consensus executes (for inspection and tests; lives until
 * detag_factors_destroy): `*batches` batches of 4 operations of 8 words each,
 *   { o0, o1, dst, keep, w0, w1, m0, m1 }:   acc = (previous acc & keep) + w0*(row[o0] & m0) + w1*(row[o1] & m1),
 *                                            row[dst] = acc,
 * o0, o1, dst = 256 * row index, w0, w1 fp32 bit patterns, keep/m0/m1 all ones or 0, the first operation of a batch
 * starting from 0.  A batch reads all its operands before it writes any row and writes in operation order.  The
 * batches in order give the same rows as the R factors in order.  `*batches` = 0 when the sequence is not run that
 * way (more than 256 workers, a factor row with more than 8 terms, rows of a step that read each other in a cycle).
 */
detag_status detag_factors_get_program(const detag_factors *f, int64_t *batches, const uint32_t **words);

/*
 * End of a round of Algorithm 1: X <- Xt - scale*G;  Xt <- X;  G <- 0,
 * with Xt the averaged model copy, G the gradient buffer and scale = alpha/R.
 * X_dev, Xt_dev: state type (X_dev may equal Xt_dev); G_dev: fp32.
 */
detag_status detag_defacto_update(detag_ctx *ctx, void *X_dev, void *Xt_dev, float *G_dev, double scale,
                                  void *stream);

/* Output of Algorithm 2: xbar[c] = (1/n) sum_i X[i,c].  xbar_dev: d floats. */
detag_status detag_mean(detag_ctx *ctx, const void *X_dev, float *xbar_dev, void *stream);

/*
 * Consensus distance ||X - 1 xbar^T||_F^2 that the proof of Theorem 3 bounds.
 * sumsq_dev: one double in device memory.  Deterministic (fixed reduction order).
 */
detag_status detag_consensus_error(detag_ctx *ctx, const void *X_dev, double *sumsq_dev, void *stream);

/*
 * detag_consensus_error for callers that cannot allocate device memory (code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the same kernels, same reduction order and same result, with the
 * per-block partial sums kept in an array that is part of the library's code
 * object (512 KiB on every GPU the library runs on, held until the process
 * ends) instead of memory owned by the context.  The call allocates and frees
 * nothing and does not synchronise.
 *   - d <= 16,777,216 (65,536 partial sums, one per 256 columns); a wider
 *     context gets DETAG_EUNSUPPORTED and nothing is enqueued.
 *   - All calls on one GPU, from every context, share that GPU's array.  Every
 *     slot a call reads it has written itself, so nothing needs clearing
 *     between calls; but two calls whose work overlaps in time on one GPU
 *     (two streams, two threads, two contexts) race and give garbage: order
 *     them on one stream or with events.
 *   - The device that is current at the call must be the one X_dev lives on.
 */
detag_status detag_consensus_error_static(detag_ctx *ctx, const void *X_dev, double *sumsq_dev, void *stream);

/*
 * Stochastic gradient of f_i(x) = 1/2 sum_c h_c (x_c - b_ic)^2 at every
 * worker's own model (the gradient query of Algorithm 2):
 *   G[i,c] = h[c]*(X[i,c] - b[i,c]) + sigma * z[i,c]
 * X_dev: state type; h_dev: fp32, length ld (shared) or n x ld (h_per_worker != 0);
 * b_dev: fp32 n x ld; G_dev: fp32 n x ld (must not overlap X).
 * Noise z: if noise_dev != NULL it is an fp32 n x ld array of standard normals;
 * else if sigma != 0 it is generated in the kernel from the counter
 * (seed, step, worker, column) with Philox-4x32-10 + Box-Muller:
 *   block q = c/4, counter = (q mod 2^32, q div 2^32, i, step), key = (seed mod 2^32, seed div 2^32),
 *   u(r) = ((r>>9)+0.5)*2^-23,  z[4q+0], z[4q+1] = sqrt(-2 ln u(r0)) * (cos, sin)(2 pi u(r1)),
 *   z[4q+2], z[4q+3] likewise from (r2, r3).
 */
detag_status detag_grad_quadratic_diag(detag_ctx *ctx, const void *X_dev, const float *h_dev,
                                       int32_t h_per_worker, const float *b_dev,
                                       const float *noise_dev, float sigma, uint64_t seed,
                                       uint32_t step, float *G_dev, void *stream);

/*
 * detag_grad_quadratic_diag followed by detag_step, as one kernel: the
 * gradient query of Algorithm 2 at the phase-start model and the phase update,
 *   G+ = h*(X - b) + sigma*z, then
 *   DETAG_VARIANT_ATC : X+ = M(X - alpha*Y);       Y+ = M(Y + G+ - G)
 *   DETAG_VARIANT_ALG2: X+ = M(X) - alpha*M(Y);    Y+ = M(Y) + G+ - G.
 * G_dev (fp32 n x ld) holds the previous gradient buffer g(k-1) on entry and
 * g(k) on return, so the caller keeps ONE gradient matrix and does not swap.
 * h_dev: fp32, length ld and shared by all workers (h_per_worker = 0), or
 * n x ld with one row per worker (h_per_worker != 0, one more streamed array);
 * b_dev: fp32 n x ld; noise is
 * always the counter-based generator of detag_grad_quadratic_diag (sigma = 0
 * turns it off).  Results are identical to the two separate calls.
 * For contexts whose rounds run on chip and K >= 1 (DETAG_EUNSUPPORTED
 * otherwise: per-round or dense path, n > 256, a worker with more than 8
 * neighbours).  On the register-resident family (detag_get_kernel) both
 * variants exist and move the same bytes (read X, Y, G, b; write X, Y, G);
 * ALG2 keeps the new gradient in LDS (n KiB per block) across the rounds.  On
 * the LDS-resident family only DETAG_VARIANT_ATC exists (its LDS holds the
 * rows of the state; DETAG_EUNSUPPORTED for ALG2: use the two separate calls).
 * X, Y, G, h, b must not overlap.
 */
detag_status detag_step_quadratic(detag_ctx *ctx, void *X_dev, void *Y_dev, float *G_dev, const float *h_dev,
                                  int32_t h_per_worker, const float *b_dev, float sigma, uint64_t seed, uint32_t step, double alpha,
                                  int32_t K, double eta, int32_t variant /* detag_variant */, void *stream);

/*
 * Gradient of f_i(x) = 1/2 ||A_i x - b_i||^2:  G[i,:] = A_i^T (A_i X[i,:] - b_i).
 * A_dev: fp32 n x m x d (row pitch d), b_dev: fp32 n x m, G_dev: fp32 n x ld.
 * Uses a context-owned scratch of n*m floats (allocated on first use).
 */
detag_status detag_grad_lstsq(detag_ctx *ctx, const void *X_dev, const float *A_dev,
                              const float *b_dev, int32_t m, float *G_dev, void *stream);

/*
 * Mini-batch gradient of multinomial logistic regression (mean cross-entropy),
 * every worker on its own batch, with bf16 MFMA contractions and fp32
 * accumulation.  A row of X holds C*F weights (class-major) then C biases, so
 * the context's d must equal C*F + C.
 *   feat_dev  : bf16 (uint16 bit patterns), n x S x F — worker i's local samples
 *   labels_dev: int32 n x S, values in [0, C)
 *   batch_dev : int32 n x B, sample indices in [0, S) for this step
 *   G_dev     : fp32 n x ld;  loss_dev: fp32 n (mean loss of each batch), may be NULL
 * Limits: C <= 10, F % 32 == 0, B % 32 == 0, B <= 256.  X must be fp32.
 * The fp32 weights and the fp32 softmax residuals are split into three bf16
 * terms each before the MFMA, so the result carries fp32 accuracy with respect
 * to the bf16 features.
 */
detag_status detag_grad_softmax_bf16(detag_ctx *ctx, const void *X_dev, const uint16_t *feat_dev,
                                     const int32_t *labels_dev, const int32_t *batch_dev,
                                     int32_t S, int32_t F, int32_t C, int32_t B, float *G_dev,
                                     float *loss_dev, void *stream);

/* Text of the last failure on this context (or of the last failed detag_create
 * on this thread when ctx is NULL).  Never NULL. */
const char *detag_last_error(const detag_ctx *ctx);

/* Library version string. */
const char *detag_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DETAG_H */
