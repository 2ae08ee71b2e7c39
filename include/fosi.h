/*
 * fosi.h -- C boundary of the MI355X (gfx950) hot path of the hybrid-order
 * optimiser: Lanczos on Hessian-vector products with full reorthogonalisation
 * (Algorithm 1), Ritz extraction of the k largest / l smallest pairs (Eq. 8),
 * the two-subspace update (Eq. 4, Eq. 12; Eq. 14 with a dual variable) and the
 * outer multiplier rule (Eq. 11, Algorithm 3).
 *
 * Conventions that hold for every call
 *   - "dev" pointers are device (HBM) addresses on the context's GPU, "host"
 *     pointers are ordinary host memory.  The caller owns every buffer it
 *     passes; the library only allocates its own scratch (a few MiB per
 *     context, plus per-operator caches stated below).
 *   - Vectors are fp32 of length n.  Matrices are fp32 column-major with a
 *     leading dimension ld >= n that is a multiple of 4 floats; matrix and
 *     vector base pointers are 16-byte aligned.  Violations return
 *     FOSI_ERR_BAD_LAYOUT.
 *   - Work is enqueued on the context's HIP stream.  fosi_lanczos (and
 *     fosi_lanczos_end, fosi_lanczos_row_sharded) block until the tridiagonal has
 *     been copied to the host; fosi_ritz solves the small eigenproblem on the host
 *     and then only enqueues; every other call only enqueues.  The two small
 *     host-to-device uploads (the Ritz coefficient block, the Newton factors when
 *     they change) go through pinned staging buffers owned by the context, so
 *     neither synchronises the stream; a call that needs a staging buffer again
 *     while its previous copy is still in flight waits for that copy alone.
 *     Host arrays passed to a call (alpha, beta, evals) are read before it returns.
 *   - No call aborts, throws or prints (host allocation failures inside the
 *     library come back as FOSI_ERR_NOMEM).  A negative status is an error and
 *     fosi_last_error(ctx) describes it.
 *   - Reductions are two-stage with a fixed order: a repeated call on the same
 *     inputs returns the same bits.
 */
#ifndef FOSI_H
#define FOSI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t fosi_status;
#define FOSI_OK                0
#define FOSI_ERR_INVALID_ARG  (-1)  /* null pointer, non-positive size, unknown enum            */
#define FOSI_ERR_BAD_LAYOUT   (-2)  /* ld < n, ld not a multiple of 4, misaligned pointer       */
#define FOSI_ERR_RANK         (-3)  /* more Ritz pairs requested than Lanczos steps available   */
#define FOSI_ERR_NONFINITE    (-4)  /* NaN/Inf met in the recurrence, or a zero Newton divisor  */
#define FOSI_ERR_HIP          (-5)  /* a HIP runtime call failed                                */
#define FOSI_ERR_NOMEM        (-6)  /* scratch allocation failed                                */
#define FOSI_ERR_CALLBACK     (-7)  /* a user hvp callback returned non-zero                    */
#define FOSI_ERR_LIMIT        (-8)  /* a size exceeds a built-in limit (see FOSI_MAX_COLS)      */

/* Largest number of matrix columns any kernel handles (Lanczos steps + 1,
 * planted rank, k + l).  Consequence for the paper's own rule for the number
 * of Lanczos steps, m = max{4 (k + l), 2 ln n} (fosi_lanczos_steps): m <= 255
 * means the rule can be followed up to k + l = 63 requested pairs; beyond
 * that fosi_lanczos returns FOSI_ERR_LIMIT for the rule's m and the caller has
 * to run fewer steps than the rule asks for. */
#define FOSI_MAX_COLS 256

typedef struct fosi_ctx fosi_ctx;   /* one GPU + one stream + scratch; not thread-safe */
typedef struct fosi_hvp fosi_hvp;   /* a curvature operator v -> H v bound to a context */

/* ---- context ---------------------------------------------------------- */

/* Creates a context on GPU `device`.  `hip_stream` is a hipStream_t passed as
 * a pointer (NULL = the default stream); the caller keeps the stream alive.
 * Launch shapes are fixed at creation; for experiments they can be overridden through environment variables
 * read here (values outside a knob's range fall back to the default):
 *   FOSI_DOT_BLOCKS   resident workgroups targeted by the transposed product (default 0: 2 per compute unit up
 *                     to 8 M rows, 1 beyond)
 *   FOSI_DOT_JB       columns per wave in that kernel: 8, 16, 32 (default 0: 8 up to 4 M rows, else 16)
 *   FOSI_COMB_ROWS / FOSI_COMB_COLS / FOSI_COMB_BLOCKS   row groups per thread and columns loaded together (one of
 *                     1x8, 1x16, 2x4, 2x8, 4x2, 4x4, 4x8, 8x2, 8x3, 8x4; default: 4x8 up to 8 M rows, 8x4 beyond)
 *                     and grid cap (0: none) of the column-combination kernel
 *   FOSI_STEP_WAVES   resident waves per compute unit aimed at by the update's fused second sweep (8)
 *   FOSI_STEP_COLS    columns of V-hat per wave in that sweep: 16, 24 or 32 (default 0: 16 up to 32 columns, else 24)
 *   FOSI_EARLY_BETA   1: beta from the Gram-Schmidt coefficients, normalisation inside the subtraction (default)
 *   FOSI_RITZ_MFMA    1: Ritz vectors on the matrix cores (default); 0: on the vector ALUs
 *   FOSI_GGN_DIRECT   1: the softmax-GGN products load their operand tiles straight into LDS where the shape allows
 *                     (default); 0: always stage them through registers */
fosi_status fosi_ctx_create(fosi_ctx** out, int device, void* hip_stream);
/* Bytes of device memory a context holds for itself to serve problems of n rows, m Lanczos steps and r_v = k + l
 * Ritz pairs (partial sums, coefficient vectors, the tridiagonal, flags); every other buffer is the caller's.  The
 * scratch is laid out for the built-in limits, so the answer is the same (about 9 MiB) for every admissible size;
 * 0 for sizes beyond the limits.  Host-only, needs no context.  Operators created by hvp_softmax_ggn*_create own
 * their work matrices in addition (stated there). */
size_t fosi_workspace_bytes(int64_t n, int m, int r_v);
fosi_status fosi_ctx_destroy(fosi_ctx* ctx);
/* Blocks until all work enqueued through this context has finished. */
fosi_status fosi_ctx_synchronize(fosi_ctx* ctx);
/* Text of the last error on this context ("" if none).  Owned by the context. */
const char* fosi_last_error(const fosi_ctx* ctx);
const char* fosi_status_string(fosi_status s);

/* ---- curvature operators: the input hvp_t of Algorithm 1 ------------------
 * The paper obtains H v from a network by automatic differentiation; these
 * operators take its place.  All of them read v_dev and write hv_dev (both fp32,
 * length n, distinct buffers) on the context's stream. */

/* H = U diag(lam) U^T + shift I.  U_dev: n x r column-major (ldu), lam_dev: r
 * fp32.  Both are read at every apply and stay owned by the caller. */
fosi_status hvp_planted_create(fosi_ctx* ctx, int64_t n, int r, const float* U_dev, int64_t ldu,
                               const float* lam_dev, float shift, fosi_hvp** out);
/* H = diag(d).  d_dev: n fp32. */
fosi_status hvp_diag_create(fosi_ctx* ctx, int64_t n, const float* d_dev, fosi_hvp** out);
/* Generalised Gauss-Newton matrix of the mean softmax cross-entropy of a linear
 * classifier, logits = X W:  H v = X^T[(diag(p_b) - p_b p_b^T)(X V)_b]_b / B with
 * V = v viewed as d x C row-major, n = d*C.  X_dev: B x d row-major, W_dev:
 * d x C row-major.  The operator caches P = softmax(X W), up to eight B x C
 * matrices of partial products and a transposed copy of X in device memory it
 * allocates (freed by hvp_destroy); X_dev is read at creation and at every apply
 * and must not change while the operator lives. */
fosi_status hvp_softmax_ggn_create(fosi_ctx* ctx, int B, int d, int C, const float* X_dev,
                                   const float* W_dev, fosi_hvp** out);
/* The same operator for a data matrix stored in bf16 (X_bf16_dev: B x d row-major, raw 16-bit
 * patterns; the operator is defined by exactly these values).  The two products run on the bf16 matrix
 * cores with fp32 accumulation; the fp32 operand of each product (V, then the softmax-Jacobian rows)
 * is split on the fly into two bf16 parts that together keep ~17 bits of it, so one application is
 * accurate to a few 1e-6 relative.  The operator additionally owns a transposed bf16 copy of X and
 * the partial results of the second product. */
fosi_status hvp_softmax_ggn_bf16_create(fosi_ctx* ctx, int B, int d, int C, const uint16_t* X_bf16_dev,
                                        const float* W_dev, fosi_hvp** out);
/* User operator (for instance a double-backward pass).  fn must enqueue its
 * work on `stream` (a hipStream_t) and return 0 on success. */
typedef int (*fosi_hvp_fn)(void* user, const float* v_dev, float* hv_dev, void* stream);
fosi_status hvp_callback_create(fosi_ctx* ctx, int64_t n, fosi_hvp_fn fn, void* user, fosi_hvp** out);
fosi_status hvp_apply(fosi_hvp* op, const float* v_dev, float* hv_dev);
fosi_status hvp_destroy(fosi_hvp* op);

/* ---- Algorithm 1: Lanczos with full reorthogonalisation ------------------- */

/* How the Gram-Schmidt line of Algorithm 1 (h <- h - D (D^T h)) is carried out. */
#define FOSI_REORTH_SINGLE      1   /* one pass against all columns: the line as printed            */
#define FOSI_REORTH_TWICE       2   /* that pass done twice                                         */
#define FOSI_REORTH_LOCAL_FULL  3   /* default: a pass against the last two columns (the only ones  */
                                    /* h is not orthogonal to in exact arithmetic), then the        */
                                    /* printed pass against all columns                             */
#define FOSI_REORTH_SELECTIVE   4   /* the printed pass, and a second one only in the steps where    */
                                    /* the first left less than reorth_eta * ||H q_i|| (the test of  */
                                    /* Daniel, Gragg, Kaufman and Stewart): a pass in fp32 storage   */
                                    /* leaves an error of ~1e-7 ||H q_i||, which only matters        */
                                    /* against a small remainder                                     */
typedef struct {
    /* 0 selects the default.  fp32 storage needs a second pass of some kind to keep Q orthonormal:
     * TWICE and LOCAL_FULL reach the same orthogonality (~1e-8), LOCAL_FULL with about half the
     * traffic.  With more than one pass the diagonal entry is the sum of the coefficients removed
     * along the current vector. */
    int32_t reorth_mode;
    /* The step count stops early (m_eff < m) when ||h after orthogonalisation||
     * <= breakdown_tol * ||H q_i||: the Krylov space is exhausted.  Default 1e-6. */
    double breakdown_tol;
    /* FOSI_GRAPH_OFF (0, default): the seven kernels of every step (default scheme) are launched one by one.
     * FOSI_GRAPH_ON (1): when the context's stream can be captured (it is not the null stream),
     * profiling is off and the operator is not a callback, the launches of the whole run are captured
     * once into a HIP graph, kept in the context and replayed for as long as the operator, sizes,
     * pointers and options stay the same; otherwise the run is launched eagerly.  Results are
     * bit-identical either way (every sum has a fixed order).  Measured on MI355X the replay is not
     * faster than eager launches (75 us per step at n = 65 536 both ways): below a few million rows
     * a step is bound by the GPU's own latency between dependent kernels, not by the host. */
    int32_t graph_mode;
    /* FOSI_REORTH_SELECTIVE only: threshold of the second pass, in (0, 1); 0 selects 1/sqrt(2), the value the
     * test's analysis asks for: a step that skips the pass multiplies the loss of orthogonality already present
     * by up to 1/eta^2 - 1, so below 1/sqrt(2) the errors can compound from step to step (measured at
     * n = 25.6 M, m = 80: max |Q^T Q - I| 3.6e-11 with the default, 7e-7 with 0.3, 6e-3 with 0.1).  Smaller
     * values are accepted for studying the scheme; other values are FOSI_ERR_INVALID_ARG. */
    double reorth_eta;
} fosi_lanczos_opts;
#define FOSI_GRAPH_OFF  0
#define FOSI_GRAPH_ON   1

/* The paper's rule for the number of Lanczos steps (paragraph introducing Algorithm 1):
 * m = max{4 (k + l), 2 ln n}, rounded up.  Host-only; returns 0 for invalid arguments. */
int32_t fosi_lanczos_steps(int64_t n, int k, int l);

/* Q_dev: n x (m+1) column-major (ldq).  On entry column 0 holds the start
 * vector (any non-zero vector: it is normalised in place); on exit columns
 * 0..m_eff-1 are the orthonormal Lanczos vectors and column m_eff (if
 * m_eff == m: the residual direction) is scratch.
 * alpha_host, beta_host: m doubles each, first m_eff valid.  beta[i] couples
 * columns i and i+1; beta[m_eff-1] is the norm of the final residual.
 * opts may be NULL (defaults).  Breakdown is not an error. */
fosi_status fosi_lanczos(fosi_ctx* ctx, fosi_hvp* op, int64_t n, int m, float* Q_dev, int64_t ldq,
                         double* alpha_host, double* beta_host, int32_t* m_eff,
                         const fosi_lanczos_opts* opts);

/* The same run in two halves, for callers that drive several contexts (parameter blocks on streams of their own)
 * from one host thread: fosi_lanczos_begin checks the arguments and enqueues the whole run without waiting for the
 * GPU; fosi_lanczos_end waits for it and delivers alpha, beta (m doubles each, m as passed to begin) and m_eff.
 * Between the two, other contexts may be used freely; on this context only fosi_lanczos_end (or fosi_ctx_destroy) may
 * follow.  The start vector, Q_dev and the operator must stay untouched until fosi_lanczos_end returns.
 * fosi_lanczos is begin followed by end.  Errors: a second begin while a run is pending, or an end without one, is
 * FOSI_ERR_INVALID_ARG; a begin that fails leaves nothing pending. */
fosi_status fosi_lanczos_begin(fosi_ctx* ctx, fosi_hvp* op, int64_t n, int m, float* Q_dev, int64_t ldq,
                               const fosi_lanczos_opts* opts);
fosi_status fosi_lanczos_end(fosi_ctx* ctx, double* alpha_host, double* beta_host, int32_t* m_eff);

/* Number of graph captures and graph replays fosi_lanczos has done on this context so far
 * (either pointer may be NULL). */
fosi_status fosi_graph_stats(fosi_ctx* ctx, int64_t* captures, int64_t* replays);

/* Number of steps of the context's last completed Lanczos run in which FOSI_REORTH_SELECTIVE took its second
 * pass (0 for the other schemes).  Host-only. */
fosi_status fosi_lanczos_second_passes(fosi_ctx* ctx, int32_t* count);

/* Algorithm 2 (row-sharded Lanczos) emulated on one GPU: the n rows are cut into `shards` contiguous
 * blocks ("virtual devices", boundaries at multiples of 64 rows).  Every sweep runs once per block on
 * that block's rows of Q (and of U for the planted operator) and leaves its partial sums in one row of
 * an exchange buffer; a separate small kernel adds the rows in rank order -- the place an all-reduce
 * takes in the distributed algorithm -- and every block continues from the summed values.  Operators
 * other than the planted one are applied to the whole vector (the algorithm's all-gather of v_i is the
 * identity when all blocks live in one memory).  Same arguments, outputs and error behaviour as
 * fosi_lanczos; 1 <= shards <= FOSI_MAX_SHARDS.  Results agree with fosi_lanczos up to the summation
 * order of the partial sums.  FOSI_REORTH_SELECTIVE is not available here (FOSI_ERR_INVALID_ARG).  Meant for
 * validating the sharded scheme, not for speed. */
#define FOSI_MAX_SHARDS 64
fosi_status fosi_lanczos_row_sharded(fosi_ctx* ctx, fosi_hvp* op, int64_t n, int m, int shards, float* Q_dev,
                                     int64_t ldq, double* alpha_host, double* beta_host, int32_t* m_eff,
                                     const fosi_lanczos_opts* opts);

/* ---- Eq. 8: Ritz extraction ------------------------------------------------ */

/* Host-only helper: eigen-decomposition of the symmetric tridiagonal matrix
 * with diagonal alpha[0..m-1] and off-diagonal beta[0..m-2].  evals: m doubles,
 * ascending.  evecs: m x m doubles, column-major, column j belongs to evals[j]
 * (may be NULL).  Touches no GPU. */
fosi_status fosi_tridiag_eigh(int m, const double* alpha, const double* beta, double* evals, double* evecs);

/* Solves the m_eff x m_eff tridiagonal problem on the host, keeps the k largest
 * (descending) then the l smallest (ascending) Ritz values and forms their Ritz
 * vectors V = Q[:, :m_eff] S on the GPU.  V_dev: n x (k+l) column-major (ldv).
 * evals_host: k+l doubles.  resid_host: k+l residual estimates
 * beta[m_eff-1] * |last component of the eigenvector| (may be NULL).
 * Needs 1 <= k+l <= m_eff, else FOSI_ERR_RANK. */
fosi_status fosi_ritz(fosi_ctx* ctx, int64_t n, int m_eff, const float* Q_dev, int64_t ldq,
                      const double* alpha_host, const double* beta_host, int k, int l,
                      float* V_dev, int64_t ldv, double* evals_host, double* resid_host);

/* ---- Eq. 4 + Eq. 12 (Eq. 14 with a dual variable): one model update --------- */

#define FOSI_CURV_SIGNED 0   /* divide by (a_j + sigma) as the equations are written */
#define FOSI_CURV_ABS    1   /* divide by (|a_j| + sigma)                            */

typedef struct {
    float alpha;      /* Newton scale                                        */
    float lr;         /* learning rate of the base optimiser (heavy ball)    */
    float momentum;   /* heavy-ball coefficient                              */
    float sigma;      /* ADMM penalty; ignored when pi_dev is NULL            */
    int32_t curv_mode;
} fosi_step_params;

/* w <- w + Delta_1 + Delta_2 with
 *   g~ = g + pi (pi = 0 if pi_dev is NULL),  c = V^T g~,
 *   Delta_1 = -alpha V (c / (a + sigma)),
 *   b <- momentum b + (g~ - V c),  o = -lr b,  Delta_2 = o - V (V^T o).
 * V_dev: n x r_v column-major (ldv), r_v = k+l >= 0 (0: plain heavy ball);
 * evals_host: r_v doubles; g_dev, pi_dev: n fp32 read-only; mom_dev (b) and
 * w_dev: n fp32, updated in place. */
fosi_status fosi_step(fosi_ctx* ctx, int64_t n, int r_v, const float* V_dev, int64_t ldv,
                      const double* evals_host, const float* g_dev, const float* pi_dev,
                      float* mom_dev, float* w_dev, const fosi_step_params* p);

/* The same update for callers that cannot allocate device memory: code running under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  No context is needed and nothing is allocated or freed, on the
 * device or through any library: the scratch memory of the update's kernels (partial sums, coefficient vectors,
 * Newton factors) is a static device array of FOSI_NOALLOC_SCRATCH_BYTES (about 2.1 MiB) that every GPU the
 * library runs on holds until the process ends; its address on a GPU is looked up once, at the first call made
 * with that GPU current (make that first call outside a capture).  Arguments, layout rules, arithmetic and results
 * are those of fosi_step (same kernels, bit-identical output); hip_stream is a hipStream_t (NULL: the default
 * stream) of the CURRENT device, to which all device pointers must belong.  Limits: r_v <= FOSI_NOALLOC_MAX_COLS,
 * else FOSI_ERR_LIMIT; errors come back as the status alone (there is no context to hold a message).  All calls on
 * one GPU share that GPU's array and it keeps the last call's contents (what must start from a defined value is
 * rewritten by a kernel at the start of each call): calls that overlap on one GPU, from several streams or
 * threads, race.  The divisors travel as a kernel argument, so evals_host is read before the call returns and no
 * host-to-device copy is enqueued. */
#define FOSI_NOALLOC_MAX_COLS       64
#define FOSI_NOALLOC_SCRATCH_BYTES  2133760
fosi_status fosi_step_noalloc(void* hip_stream, int64_t n, int r_v, const float* V_dev, int64_t ldv,
                              const double* evals_host, const float* g_dev, const float* pi_dev,
                              float* mom_dev, float* w_dev, const fosi_step_params* p);

/* Same update with AdamW as the base first-order optimiser (the optimiser of the paper's experiments,
 * Section IV hyper-parameter paragraph).  The optimiser's descent vector is
 *   o = -lr ( m^ / (sqrt(v^) + eps) + weight_decay w ),
 * m, v the running moments of x = g~ - V c with bias corrections for step_index (1-based), and
 *   Delta_2 = o - V (V^T o)   (the decoupled decay is part of the vector that is re-projected).
 * exp_avg_dev, exp_avg_sq_dev: n fp32 moments, updated in place; work_dev: n fp32 scratch owned by the
 * caller (receives o); w_dev updated in place.  With r_v = 0 this is textbook AdamW. */
typedef struct {
    float alpha;          /* Newton scale */
    float lr, beta1, beta2, eps, weight_decay;
    float sigma;          /* ADMM penalty; ignored when pi_dev is NULL */
    int32_t curv_mode;
} fosi_adamw_params;
fosi_status fosi_step_adamw(fosi_ctx* ctx, int64_t n, int r_v, const float* V_dev, int64_t ldv,
                            const double* evals_host, const float* g_dev, const float* pi_dev,
                            float* exp_avg_dev, float* exp_avg_sq_dev, float* work_dev, float* w_dev,
                            int64_t step_index, const fosi_adamw_params* p);

/* ---- Algorithm 3 / Eq. 11: outer multiplier rule ---------------------------- */

/* Start of an outer iteration: w_anchor = w_a + pi / sigma; w_a = w_anchor. */
fosi_status fosi_admm_begin(fosi_ctx* ctx, int64_t n, float sigma, const float* pi_dev,
                            float* w_anchor_dev, float* wa_dev);
/* End of an outer iteration: pi <- pi + sigma (w_a - w_anchor). */
fosi_status fosi_admm_end(fosi_ctx* ctx, int64_t n, float sigma, const float* w_anchor_dev,
                          const float* wa_dev, float* pi_dev);

/* ---- measurement aid ---------------------------------------------------------
 * Not a step of the method (no passage of the paper defines it): a memory-only model of a sweep.
 * Reads cols_in columns of A (device, fp32 column-major, lda) and writes cols_out columns of B (device, ldb) with
 * the streaming loads, streaming stores and workgroup tiling of the library's own sweeps and no arithmetic beyond
 * one add per loaded value; column w of B receives (w + 1) * (sum of the columns of A), or zeros when cols_in == 0
 * (write-only), and nothing is written when cols_out == 0 (read-only; B_dev may then be NULL).  Timed through the
 * FOSI_PROF_TRAFFIC_MODEL class it states what the device's memory system gives to a given mix of read and
 * written columns (bench.py --traffic-model): the yardstick for the kernels whose traffic is that mix -- the Ritz
 * vectors (m read, k + l written) and the update's sweeps (k + l + 2 read, 1 written).
 * n: rows, a positive multiple of 4.  Only enqueues.  FOSI_ERR_INVALID_ARG / FOSI_ERR_BAD_LAYOUT as elsewhere. */
fosi_status fosi_traffic_model(fosi_ctx* ctx, int64_t n, const float* A_dev, int64_t lda, int cols_in, float* B_dev,
                               int64_t ldb, int cols_out);

/* ---- per-kernel timing (opt-in) --------------------------------------------
 * When enabled, every launch of the kernels listed below is bracketed by HIP
 * events on the context's stream.  fosi_profile_read synchronises and returns
 * the launch count, the summed duration and the summed algorithmic bytes of
 * one kernel class since the last reset. */
#define FOSI_PROF_HVP_PROJECT   0   /* planted operator: coefficients U^T v            */
#define FOSI_PROF_HVP_EXPAND    1   /* planted operator: shift v + U (lam . coeff)     */
#define FOSI_PROF_REORTH_DOT    2   /* Gram-Schmidt: Q^T h                             */
#define FOSI_PROF_REORTH_SUB    3   /* Gram-Schmidt: h - Q c, ||.||^2                  */
#define FOSI_PROF_NORMALISE     4   /* q = h / beta                                    */
#define FOSI_PROF_RITZ_VECTORS  5   /* V = Q S                                         */
#define FOSI_PROF_STEP          6   /* all kernels of one fosi_step                    */
#define FOSI_PROF_ADMM          7   /* multiplier rule kernels                         */
#define FOSI_PROF_HVP_GGN       8   /* softmax-GGN operator, whole apply; the "bytes"   */
                                    /* field returns its GEMM flops (4 B d C) instead  */
#define FOSI_PROF_HVP_OTHER     9   /* diagonal / callback operators                   */
/* The three sweeps of fosi_step one by one.  Recorded only when the whole-step class is NOT selected (select them
 * with FOSI_PROF_ONLY): the step's kernels carry either the one bracket or these three. */
#define FOSI_PROF_STEP_PROJECT 10   /* c = V^T (g + pi)                                */
#define FOSI_PROF_STEP_COMPLEMENT 11 /* b <- mu b + (g + pi) - V c, e = V^T b (fused)   */
#define FOSI_PROF_STEP_APPLY   12   /* w <- w - lr b - V d                             */
#define FOSI_PROF_TRAFFIC_MODEL 13  /* fosi_traffic_model                              */
#define FOSI_PROF_NUM          14
/* on = 0: off; 1: every class; FOSI_PROF_ONLY(c) [| FOSI_PROF_ONLY(c2) ...]: only those classes.  Two events
 * around a kernel cost about 5 us of stream time each on MI355X (the stream drains at every event), so a
 * timed run that must not be disturbed selects the one class it needs. */
#define FOSI_PROF_ONLY(kernel_class) (1 << ((kernel_class) + 1))
fosi_status fosi_profile_enable(fosi_ctx* ctx, int on);
fosi_status fosi_profile_reset(fosi_ctx* ctx);
fosi_status fosi_profile_read(fosi_ctx* ctx, int kernel_class, int64_t* launches, double* total_ms,
                              double* algorithmic_bytes);

#ifdef __cplusplus
}
#endif
#endif /* FOSI_H */
