/*
 * pdadmm.h - C ABI of the MI355X (gfx950) implementation of one pdADMM-G / pdADMM-G-Q
 * iteration over all layers of a graph-augmented MLP (arXiv 2105.09837).
 *
 * Conventions
 *  - "DEVICE" pointers are HIP device memory owned by the caller; "HOST" pointers are
 *    ordinary host memory. The library never allocates or frees device memory: all state
 *    lives in the caller's workspace (pdadmm_workspace_bytes / pdadmm_init).
 *  - The paper's n x |V| matrices are stored node-major, row-major [|V|, n] fp32 (the same
 *    bytes as the paper's matrix in column-major). W_l is row-major [n_l, n_{l-1}].
 *  - Layers are numbered 1..L as in the paper. p_1 = X (the augmented features) is fixed.
 *  - Every call returns a pdadmm_status; pdadmm_last_error(ctx) gives a text for the last
 *    failure on that context. Nothing throws or aborts across this boundary. A context is
 *    not thread-safe. After PDADMM_EHIP the context must be destroyed.
 *  - Kernels are enqueued on the stream given at init / in the call (a hipStream_t passed
 *    as void*; NULL = the default stream). pdadmm_iterate is asynchronous for pdADMM-G;
 *    for pdADMM-G-Q it waits for one 4-byte-per-layer flag copy per pair of backtracking rounds.
 *  - Calls that have no context (or fail before one exists) leave their reason in a per-thread
 *    text that pdadmm_last_error(NULL) returns.
 */
#ifndef PDADMM_H
#define PDADMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pdadmm_ctx pdadmm_ctx;

typedef enum {
  PDADMM_OK = 0,
  PDADMM_EINVAL = 1,      /* bad argument (NULL, size, range, alignment) */
  PDADMM_ENOMEM = 2,      /* workspace smaller than pdadmm_workspace_bytes() */
  PDADMM_EHIP = 3,        /* a HIP runtime call failed */
  PDADMM_EBACKTRACK = 4,  /* bt_max_trials exceeded in a p- or W-update */
  PDADMM_ENONFINITE = 5   /* a norm that drives a step size became NaN/Inf */
} pdadmm_status;

/* Problem 2 / Problem 3 of the paper plus the conventions the paper leaves open. */
typedef struct {
  int32_t n_nodes;         /* |V| */
  int32_t n_layers;        /* L >= 1 */
  const int32_t* dims;     /* HOST, dims[0..L] = n_0..n_L (read during the call only) */
  float rho, nu;           /* penalties of L_rho (Section 3.2), both > 0 */
  int32_t quantize;        /* 0: pdADMM-G; 1: pdADMM-G-Q, p_l (l >= 2) restricted to Delta; 2: the variant of
                              Appendix B that also projects every updated q_l onto Delta */
  float q_lo, q_hi;        /* Delta = { q_lo + i*(q_hi-q_lo)/(q_levels-1) }, i = 0..q_levels-1 */
  int32_t q_levels;        /* 2..65536; up to 256 the library keeps p_l as one byte per element, above as two */
  int32_t fista_iters;     /* fixed number of FISTA steps for z_L (Appendix A); e.g. 20 */
  float bt_eta;            /* backtracking growth factor (> 1), e.g. 2. Every p- and W-update starts at the
                              previous tau (theta) divided by bt_eta and multiplies by bt_eta until the
                              condition of Appendix A holds. In -Q, where each trial costs a product, the
                              smaller start value is probed with back-off: after a probe that was rejected
                              the next 1, 2, 4, ... (at most 16) updates start at the previous tau itself */
  float tau0, theta0;      /* initial tau_l, theta_l, e.g. 1 */
  int32_t bt_max_trials;   /* cap per update, e.g. 64 */
  int32_t refresh_every;   /* recompute W_l p_l + b_l - z_l from scratch every k iterations; 0 = never */
  float leaky_slope;       /* activation f(z) = z (z > 0), leaky_slope * z otherwise; 0 = ReLU (Section 5.1);
                              in [0, 1): leaky ReLU (named in Section 4 as satisfying the assumption) */
  int32_t use_graph;       /* 1: pdADMM-G iterations are captured once as a HIP graph and replayed on a stream
                              of the library's own, ordered against `stream` by events (helps small,
                              launch-bound models). Ignored for -Q, while pdadmm_timing is on and when
                              refresh_every > 0 */
  int32_t bt_probe_backoff;/* -Q only. 1: the smaller start value tau/bt_eta is probed with the back-off described
                              at bt_eta. 0: plain schedule, every p-update starts at the previous tau divided by
                              bt_eta exactly as in pdADMM-G (one more product per update once tau has settled).
                              Appendix A fixes only the acceptance condition; both schedules meet it */
  int32_t risk_kind;       /* R(z_L; y) of Problem 2: 0 = cross-entropy (Section 5.1), z_L by FISTA;
                              1 = least squares 1/2 ||z_j - e_{y_j}||^2 summed over labelled nodes (Section 3.1
                              admits any convex continuous risk), z_L = (e_y + nu (W_L p_L + b_L)) / (1 + nu) in
                              closed form (the z_L line of Appendix A 'update z' with this R) */
} pdadmm_config;

/* Terms of the augmented Lagrangian L_rho (Section 3.2). */
typedef struct {
  double risk;       /* R(z_L; y): cross-entropy summed over labelled nodes */
  double lin_pen;    /* (nu/2) sum_l ||z_l - W_l p_l - b_l||^2 */
  double act_pen;    /* (nu/2) sum_{l<L} ||q_l - f(z_l)||^2 */
  double dual_lin;   /* sum_{l<L} <u_l, p_{l+1} - q_l> */
  double dual_quad;  /* (rho/2) sum_{l<L} ||p_{l+1} - q_l||^2 */
  double F;          /* risk + lin_pen + act_pen (objective of Problem 2) */
  double L_rho;      /* F + dual_lin + dual_quad */
} pdadmm_objective_terms;

/* Variables addressable by pdadmm_get_var / pdadmm_set_var. */
enum {
  PDADMM_VAR_P = 0,      /* p_l, l = 1..L (l = 1 is read-only), [N, n_{l-1}] */
  PDADMM_VAR_W = 1,      /* W_l, [n_l, n_{l-1}] */
  PDADMM_VAR_B = 2,      /* b_l, [n_l] */
  PDADMM_VAR_Z = 3,      /* z_l, [N, n_l] */
  PDADMM_VAR_Q = 4,      /* q_l, l = 1..L-1, [N, n_l] */
  PDADMM_VAR_U = 5,      /* u_l, l = 1..L-1, [N, n_l] */
  PDADMM_VAR_TAU = 6,    /* tau_l, l = 2..L: one HOST double */
  PDADMM_VAR_THETA = 7,  /* theta_l, l = 1..L: one HOST double */
  PDADMM_VAR_PIDX = 8,   /* get only, -Q: indices of p_l in Delta, uint8 (uint16 if q_levels > 256) [N, n_{l-1}], l = 2..L (this is how the library
                            keeps p_l in -Q; PDADMM_VAR_P forms the values Delta[index] on the way out and takes
                            the indices of the nearest members on the way in) */
  /* (diagnostics) read-only internals */
  PDADMM_VAR_RESID = 9,  /* carried W_l p_l + b_l - z_l, [N, n_l] */
  PDADMM_VAR_GRAD_P = 10,/* last gradient of phi in p_l, [N, n_{l-1}], l = 2..L */
  PDADMM_VAR_GRAD_W = 11,/* last gradient of phi in W_l, [n_l, n_{l-1}] */
  PDADMM_VAR_PROBE = 12  /* (diagnostics; part of a -Q checkpoint) l = 2..L: two HOST int32 {wait, left}: back-off
                            state of the tau search */
};

/* Phases of Algorithm 1 as this library groups them (pdadmm_step_phase). */
enum { PDADMM_PHASE_P = 0, PDADMM_PHASE_W = 1, PDADMM_PHASE_BZQU = 2 };

/*
 * Renormalised adjacency (Section 5.1): A~ = (D+I)^(-1/2) (A+I) (D+I)^(-1/2), D_ii = sum_j A_ij.
 * In : HOST CSR pattern of the symmetric binary A without self-loops (rowptr[n+1], colidx[nnz],
 *      columns ascending within a row).
 * Out: HOST CSR of A~ with the diagonal inserted: out_rowptr[n+1], out_colidx[nnz+n] ascending,
 *      out_vals[nnz+n] = fp32(1/sqrt((d_i+1)(d_j+1))) computed in fp64. Caller owns all arrays.
 * Errors: EINVAL on NULL, negative n, non-monotone rowptr, column out of range or a self-loop.
 */
pdadmm_status pdadmm_normalize_adj(int32_t n, const int32_t* rowptr, const int32_t* colidx,
                                   int32_t* out_rowptr, int32_t* out_colidx, float* out_vals);

/*
 * Multi-hop augmentation (Sections 3.1, 5.1): X_aug = [X | A~X | ... | A~^hops X] along features.
 * All pointers DEVICE. rowptr[n+1], colidx[nnz], vals[nnz] = CSR of A~; X is [n, d] row-major;
 * X_aug is [n, (hops+1)*d] row-major, written entirely. Rounding is fixed: each product is rounded
 * to fp32 and added to an fp32 accumulator starting at +0 in CSR order (no fused multiply-add), so
 * the result is reproducible bit for bit. Asynchronous on `stream`. hops >= 0, d >= 1.
 * nnz = number of stored entries (needed to validate nothing on the device; pass rowptr[n]).
 */
pdadmm_status pdadmm_augment(int32_t n, int64_t nnz, const int32_t* rowptr, const int32_t* colidx,
                             const float* vals, const float* X, int32_t d, int32_t hops,
                             float* X_aug, void* stream);

/*
 * Projection onto the uniform set Delta (Section 3.3, Appendix B): elementwise
 * argmin_{delta in Delta} |delta - v|. DEVICE in v[count]; DEVICE out idx[count] (uint8; uint16 if levels > 256) and/or
 * val[count] (either may be NULL). step = (hi-lo)/(levels-1) in fp32; t = (v-lo)/step;
 * idx = clamp(round-half-even(t), 0, levels-1); delta = lo + idx*step (product, then sum, each
 * rounded to fp32). NaN maps to index 0. levels in 2..65536 (the paper's 8- and 16-bit cases,
 * Section 5.5, are 256 and 65536). Asynchronous on `stream`.
 */
pdadmm_status pdadmm_quantize(const float* v, int64_t count, float lo, float hi, int32_t levels,
                              void* idx, float* val, void* stream);

/* ------------------------------------------------------------------------------------------------
 * DIAGNOSTICS. The entry points and variable kinds marked "diagnostics" below (pdadmm_gemm_nt/_tn,
 * pdadmm_step_phase, pdadmm_timing/_read, PDADMM_VAR_RESID / GRAD_P / GRAD_W / PROBE) exist for the
 * tests, the benchmark and the profiles; a training loop needs none of them.
 * ------------------------------------------------------------------------------------------------ */

/*
 * (diagnostics) Dense fp32 products on the matrix cores, exposed for tests and micro-benchmarks of the kernels
 * that carry the layer updates (the n_l x n_{l-1} x |V| products named in Section 3.2).
 *   pdadmm_gemm_nt: C[M,N] = A[M,K] * B[N,K]^T         (row-major, leading dimensions in floats)
 *   pdadmm_gemm_tn: C[M,N] = alpha * A[K,M]^T * B[K,N]  with the K range split in `splitk` parts
 *                   that are summed in a fixed order; `part` is DEVICE scratch of at least
 *                   splitk*M*ldc floats.
 * All pointers DEVICE. Asynchronous on `stream`. EINVAL on non-positive sizes or ld < width.
 */
pdadmm_status pdadmm_gemm_nt(int32_t M, int32_t N, int32_t K, const float* A, int32_t lda,
                             const float* B, int32_t ldb, float* C, int32_t ldc, void* stream);
pdadmm_status pdadmm_gemm_tn(int32_t M, int32_t N, int32_t K, float alpha, const float* A, int32_t lda,
                             const float* B, int32_t ldb, float* C, int32_t ldc, int32_t splitk,
                             float* part, void* stream);

/*
 * pdadmm_gemm_tn for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc. The partial products of the K chunks live in a device
 * array that is part of the library image (PDADMM_STATIC_SCRATCH_FLOATS floats = 64 MiB, held by every
 * GPU the library runs on until the process ends) instead of a caller buffer. Arguments and result are
 * those of pdadmm_gemm_tn without `part` (same kernels, same chunking, same order of additions: the
 * results are equal bit for bit). EINVAL, with a text in pdadmm_last_error(NULL), also when
 * chunks * M * ldc exceeds the array (chunks = number of K chunks actually used, <= splitk).
 * The call allocates nothing: no hipMalloc/hipFree and no allocating library routine. Nothing in the
 * array has to start at zero (every element that is summed is written by the same call first). All
 * calls on one GPU share that GPU's array: calls that overlap in time on one GPU race; calls on one
 * stream, or ordered by events, do not.
 */
#define PDADMM_STATIC_SCRATCH_FLOATS (16u * 1024u * 1024u)
pdadmm_status pdadmm_gemm_tn_static(int32_t M, int32_t N, int32_t K, float alpha, const float* A, int32_t lda,
                                    const float* B, int32_t ldb, float* C, int32_t ldc, int32_t splitk,
                                    void* stream);

/* Bytes of DEVICE workspace pdadmm_init needs for this configuration (0 if it is invalid). */
size_t pdadmm_workspace_bytes(const pdadmm_config* cfg);

/*
 * Create a context and the forward-consistent starting point of Algorithm 1:
 * p_1 = X_aug; z_l = W_l p_l + b_l; q_l = f(z_l); p_{l+1} = q_l (projected onto Delta for -Q; with
 * quantize = 2 q_l is projected as well);
 * u_l = 0; tau_l = tau0, theta_l = theta0.
 *  workspace: DEVICE, >= pdadmm_workspace_bytes(cfg), 256-byte aligned (4 KiB for the best rate of the streaming
 *             kernels: every array is placed at a multiple of 4 KiB from its start), owned by the caller and kept
 *             alive until pdadmm_destroy. X_aug [N, n_0], labels [N] int32 in [0, n_L),
 *             train_mask [N] uint8 or NULL (= every node labelled), W0[l-1] [n_l, n_{l-1}],
 *             b0[l-1] [n_l]: all DEVICE, copied during the call (the caller may free them afterwards).
 *  W0, b0: HOST arrays of L DEVICE pointers.
 *  streams, n_streams: HOST array of 0, 1 or 2 hipStream_t (as void*). streams[0] (NULL or n_streams = 0: the
 *             default stream) carries the iteration. streams[1], if given, must be another stream of the same
 *             (default) priority: work of an iteration that does not depend on the main sequence is enqueued there
 *             between event-ordered forks and joins - the W-update of layer 1, which needs nothing from the
 *             p-updates (p_1 = X is fixed), beside the p-updates of the layers above, and the z_L-update beside the
 *             fused z/q/u pass of the hidden layers (Algorithm 1: the updates of different layers are independent
 *             within a phase). Results are the same bit for bit with one stream and with two. Every call that
 *             synchronises waits for both.
 * The call synchronises streams[0] before returning.
 * Errors: EINVAL (bad config, NULL pointer, unaligned workspace) and ENOMEM (workspace too small) leave
 * *out = NULL. A HIP failure after the context exists returns EHIP with *out set: read
 * pdadmm_last_error(*out), then pdadmm_destroy(*out).
 */
pdadmm_status pdadmm_init(pdadmm_ctx** out, const pdadmm_config* cfg, void* workspace, size_t workspace_bytes,
                          const float* X_aug, const int32_t* labels, const uint8_t* train_mask,
                          const float* const* W0, const float* const* b0, void* const* streams, int32_t n_streams);

/*
 * Greedy layer-wise training (Section 3.2, the paragraph after Algorithm 1; Section 5.3 trains 2, then
 * 5, then all 10 layers): start a deeper model from a trained shallower one. A new context is set up
 * exactly as by pdadmm_init, except that layer l of the new model takes W_l, b_l from layer
 * from_layer[l-1] of the context `from` where that entry is positive (that layer must have the same
 * n_{l-1} and n_l), and from the caller's W0[l-1], b0[l-1] where it is 0. Which layers are carried over
 * is the caller's schedule (the paper fixes none); the state is the forward-consistent start of the
 * new weights, step sizes start again at tau0, theta0.
 *  from:       context with the same n_nodes; its stream is synchronised first; it stays valid and
 *              unchanged, and may be destroyed afterwards.
 *  from_layer: HOST int32 [n_layers]. W0, b0: HOST arrays of n_layers DEVICE pointers; entries of
 *              carried-over layers are ignored (NULL allowed); both may be NULL if every layer is
 *              carried over. Everything else as for pdadmm_init, the errors too (EINVAL also for a
 *              source layer out of range or of another shape).
 */
pdadmm_status pdadmm_grow_layers(pdadmm_ctx** out, const pdadmm_config* cfg, void* workspace, size_t workspace_bytes,
                                 const float* X_aug, const int32_t* labels, const uint8_t* train_mask,
                                 pdadmm_ctx* from, const int32_t* from_layer, const float* const* W0,
                                 const float* const* b0, void* const* streams, int32_t n_streams);

/*
 * Copy a variable in or out. `layer` is the paper's l. The buffer is dense (leading dimension =
 * width) and may be HOST or DEVICE memory, except TAU/THETA (HOST double) and PROBE (HOST int32[2]).
 * Both calls synchronise.
 * set_var of P in -Q mode (and of Q with quantize = 2) projects the values onto Delta. After any
 * set_var the carried residual W_l p_l + b_l - z_l is recomputed from scratch at the next iteration.
 * A checkpoint is every P (l >= 2), W, B, Z, Q, U, TAU, THETA (and PROBE in -Q); written into a fresh
 * context of the same configuration it continues the run (to rounding: the carried residual is rebuilt).
 */
pdadmm_status pdadmm_set_var(pdadmm_ctx* ctx, int32_t kind, int32_t layer, const void* src);
pdadmm_status pdadmm_get_var(pdadmm_ctx* ctx, int32_t kind, int32_t layer, void* dst);

/* Run n_iters iterations of Algorithm 1 (phases p, W, b, z, q, u; every phase over all layers). */
pdadmm_status pdadmm_iterate(pdadmm_ctx* ctx, int32_t n_iters);

/* (diagnostics) Run one phase group of the current iteration (iterate = P, W, BZQU in this order). */
pdadmm_status pdadmm_step_phase(pdadmm_ctx* ctx, int32_t phase);

/* Wait for all enqueued work; report sticky device-side errors (EBACKTRACK, ENONFINITE). */
pdadmm_status pdadmm_sync(pdadmm_ctx* ctx);

/* L_rho and its terms, evaluated from the variables (W_l p_l + b_l is recomputed). Synchronises. */
pdadmm_status pdadmm_objective(pdadmm_ctx* ctx, pdadmm_objective_terms* out);

/* sqrt(sum_l ||p_{l+1} - q_l||_F^2) (Algorithm 1, residual line) and, if per_layer != NULL, the L-1
 * per-layer norms (HOST). Synchronises. */
pdadmm_status pdadmm_residual(pdadmm_ctx* ctx, double* total, double* per_layer);

/*
 * Forward pass of the model with the current W_l, b_l (Problem 1, Section 3.1: p_1 = X,
 * p_{l+1} = f(W_l p_l + b_l), output W_L p_L + b_L) and the class it predicts per node, the first
 * maximum of the output row. The ADMM variables are not touched; the pass runs through the product
 * scratch of the iteration, so it must not be called between the phases of pdadmm_step_phase.
 *  pred:   DEVICE int32 [N] or NULL; logits: DEVICE fp32 [N, n_L] dense or NULL;
 *  mask:   DEVICE uint8 [N] or NULL: nodes counted for the accuracy (NULL = every node);
 *  accuracy: HOST or NULL: share of counted nodes whose prediction equals the label given at init.
 * Synchronises.
 */
pdadmm_status pdadmm_predict(pdadmm_ctx* ctx, int32_t* pred, float* logits, const uint8_t* mask, double* accuracy);

/* HOST outputs, each L entries or NULL: tau_l (entry 0 unused), theta_l, trials used by the last
 * p- and W-update. r_drift (or NULL): relative L2 distance between the carried and a freshly
 * computed W_l p_l + b_l - z_l over all layers. p_products (or NULL, L entries): number of
 * step-direction products W_l g / W_l d computed for layer l since init (one per iteration for
 * pdADMM-G, one per backtracking trial for -Q). Synchronises. */
pdadmm_status pdadmm_stats(pdadmm_ctx* ctx, double* tau, double* theta, int32_t* p_trials,
                           int32_t* w_trials, double* r_drift, int64_t* p_products);

/* Launch plan the context was built with (HOST outputs, each may be NULL). fused_updates: bit 0 set if
 * the p-step and the residual update r -= Wg/tau are applied in the epilogues of the dense products
 * with the step size guessed ahead (the previous one, or the previous one divided by bt_eta while the
 * step size is still falling) and corrected by a separate pass only when the
 * backtracking rule picks another one (pdADMM-G with enough product tiles to fill the chip); bit 1
 * set if the same holds for r -= Gp/theta and its column sums (both variants, same size condition).
 * A clear bit means separate streaming kernels apply that update. wgrad_split (L entries): number of
 * node-range chunks the r p^T product of each layer is split into. wtrial_split: number of chunks the
 * contraction of the G p products is split into (1 = not split). p_bytes: bytes per element in which p_l
 * (l >= 2) is resident: 4 (fp32) for pdADMM-G; 1 for -Q (2 if q_levels > 256), where p_l is a member of Delta and
 * only its index is kept (Appendix B, last paragraph; the values are formed where they are consumed: in the operand loads of the
 * products and in the streaming kernels). Does not synchronise. */
pdadmm_status pdadmm_plan_info(pdadmm_ctx* ctx, int32_t* fused_updates, int32_t* wgrad_split, int32_t* wtrial_split,
                               int32_t* p_bytes);

/*
 * (diagnostics) Per-launch timing with HIP events recorded on the context's stream around the launches of the
 * selected kernel classes (bit i of class_mask = class i; 0 switches timing off and drops pending
 * records). Classes: 0 p-gradient product (W^T r, fused gradient), 1 step-direction products
 * (W g / W d and G p), 2 W-gradient product (r p^T, split over nodes), 3 its partial-sum reduce,
 * 4 step-size selection, 5 p-step, 6 W-step, 7 residual update + column sums, 8 b-step,
 * 9 fused z/q/u update, 10 z_L-update (FISTA, or the closed form of the least-squares risk), 11 -Q trial
 * projection, 12 -Q residual update r += W d after the search, 13 residual refresh.
 * pdadmm_timing_read synchronises, adds up the elapsed milliseconds and the number of launches per
 * class since the last read into HOST arrays of n_classes >= 14 entries, and clears the records.
 */
#define PDADMM_N_TIMING_CLASSES 14
pdadmm_status pdadmm_timing(pdadmm_ctx* ctx, uint32_t class_mask);
pdadmm_status pdadmm_timing_read(pdadmm_ctx* ctx, double* ms, int64_t* launches, int32_t n_classes);

/* Text of the last failure on this context; with ctx = NULL, of the calling thread's last failed call
 * that had no context (pdadmm_init before a context exists, pdadmm_workspace_bytes, the stand-alone
 * kernels). The pointer stays valid until the next failing call on the same context / thread. */
const char* pdadmm_last_error(const pdadmm_ctx* ctx);
void pdadmm_destroy(pdadmm_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* PDADMM_H */
