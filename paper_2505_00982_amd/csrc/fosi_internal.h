// Internal declarations shared by the translation units of libfosi_hip.
// Nothing here is part of the public boundary (see include/fosi.h).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <string>
#include <vector>

#include "fosi.h"

namespace fosi {

constexpr int kThreads = 256;          // every streaming kernel uses 4 wavefronts of 64 lanes
constexpr int kMaxCols = FOSI_MAX_COLS;
constexpr int kMaxDotSlots = 4096;     // row slots (gridDim.x) of the transposed product
constexpr int kMaxShards = FOSI_MAX_SHARDS;
constexpr int kMaxNormSlots = 32768;   // blocks of the column-combination kernel that emit ||.||^2 partials

struct ProfRecord {
    int cls;
    double bytes;
    hipEvent_t start, stop;
};

struct Tunables {
    int dot_target_blocks;    // workgroups launched by the transposed product (it grid-strides over rows)
    int dot_slot_cols;        // columns per wave in that kernel: 8, 16 or 32; 0 = chosen from the row count
    int comb_rows_per_thread; // RPT: float4 row groups per thread in the column-combination kernel
    int comb_cols_unroll;     // CU: columns loaded together in that kernel
    int comb_max_blocks;      // cap on that kernel's grid (it grid-strides over row tiles); 0 = no cap
    int early_beta;           // 1 (default): 'local_full' runs take beta from the coefficients and normalise inside the subtraction
    int ritz_mfma;            // 1 (default): Ritz vectors on the matrix cores in 16-wide column blocks; 0: vector ALUs
    int step_waves_per_cu;    // resident wavefronts per CU aimed at by the fused second sweep of the update
    int step_cols_per_wave;   // columns of V-hat a wave of that sweep keeps in registers: 16, 24 or 32; 0 = chosen by width
    int ggn_direct = 1;              // softmax-GGN products: operand tiles loaded straight into LDS (0: staged through registers)
};

// Device scratch layout (one allocation per context).
struct Scratch {
    double* partials;      // kMaxDotSlots x (kMaxCols + 1)
    double* norm_partials; // 3 * kMaxNormSlots
    double* coef_a;        // kMaxCols + 1  (first Gram-Schmidt pass / operator coefficients)
    double* coef_b;        // kMaxCols + 1  (second pass)
    double* coef_c;        // kMaxCols + 1  (update-rule coefficients)
    double* coef_h;        // kMaxCols + 1  (planted operator)
    double* scal;          // 8 scalars: [0] = 1/beta, [1] = 1/||v||, [2..3] = 1, [4..5] = -alpha~, -beta~
    double* loc;           // 8 scalars: alpha~, beta~, ||H q||^2 of the local (two-column) pass
    double* alpha;         // kMaxCols
    double* beta;          // kMaxCols
    double* hnorm;         // kMaxCols
    double* newton;        // kMaxCols: alpha / (a_j + sigma)
    float* S;              // kMaxCols x kMaxCols Ritz coefficient block
    int* flags;            // [0] stop flag (1 = breakdown, 2 = non-finite), [1] completed steps, [2] arrival counter
                           // of the second reduction stage (zero between launches)
    double* xchg;          // kMaxShards x (kMaxCols + 1): per-shard coefficient partials (row-sharded emulation)
    double* xchg3;         // kMaxShards x 3: per-shard {||.||^2, local dots}
};

}  // namespace fosi

struct fosi_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    void* scratch_base = nullptr;
    size_t scratch_bytes = 0;
    fosi::Scratch s{};
    fosi::Tunables tun{};
    std::string last_error;
    bool prof_on = false;
    int prof_mask = 1;                  // 1: every kernel class; else bit (class + 1) selects a class
    bool prof_open = false;             // the last prof_begin recorded a start event
    std::vector<fosi::ProfRecord> prof;
    std::vector<hipEvent_t> event_pool;
    // pinned host staging for the two small uploads (Ritz coefficient block S, Newton factors): an asynchronous copy
    // from it needs no stream synchronisation; the event tells when the buffer may be rewritten
    float* stage_S = nullptr;           // kMaxCols x 64 floats
    double* stage_newton = nullptr;     // kMaxCols doubles
    hipEvent_t stage_S_done = nullptr, stage_newton_done = nullptr;
    bool stage_S_busy = false, stage_newton_busy = false;
    double newton_cache[FOSI_MAX_COLS] = {0};   // host copy of what `s.newton` holds
    int newton_cached = 0;              // number of valid entries in newton_cache
    // HIP graph of the last captured Lanczos run and what it was captured for
    struct GraphKey {
        const void* op = nullptr;
        const void* Q = nullptr;
        int64_t n = 0, ldq = 0;
        int m = 0, mode = 0;
        double tol = 0.0, eta = 0.0;
        bool operator==(const GraphKey& o) const {
            return op == o.op && Q == o.Q && n == o.n && ldq == o.ldq && m == o.m && mode == o.mode && tol == o.tol &&
                   eta == o.eta;
        }
    } graph_key;
    hipGraphExec_t graph_exec = nullptr;
    bool graph_unavailable = false;     // the stream refused capture once: do not try again
    int64_t graph_replays = 0, graph_captures = 0;
    int sm_count = 256;
    int pending_m = 0;                  // steps of the Lanczos run enqueued by fosi_lanczos_begin and not yet collected
    double reorth_eta = 0.70710678118654752;   // 'selective' Gram-Schmidt scheme: threshold of the run being enqueued
    int second_passes = 0;              // ... and how many steps of the last completed run took the second pass
};

struct fosi_hvp {
    enum Kind { PLANTED, DIAG, GGN, CALLBACK } kind;
    fosi_ctx* ctx;
    int64_t n;
    // planted
    int r = 0;
    const float* U = nullptr;
    int64_t ldu = 0;
    const float* lam = nullptr;
    float shift = 0.f;
    // diag
    const float* d = nullptr;
    // ggn
    int B = 0, dim = 0, C = 0;
    const float* X = nullptr;
    const float* W = nullptr;
    float* P = nullptr;     // B x C softmax probabilities
    float* Z = nullptr;     // B x C work
    float* XT = nullptr;    // fp32 path: d x ldxt transposed copy of X (owned), so that both products stage k-major tiles
    int ldxt = 0;
    bool bf16 = false;      // data matrix given in bf16: split-operand bf16 matrix-core path
    const unsigned short* Xb = nullptr;   // B x d bf16 (caller's)
    unsigned short* XTb = nullptr;        // d x B bf16 (transposed copy, owned)
    float* Y2 = nullptr;                  // split-K partials of the second product (owned)
    unsigned short* S1 = nullptr;         // bf16 (hi, lo) pair of the first product's fp32 operand, C x d each (owned)
    unsigned short* S2 = nullptr;         // ... of the second product's, C x B each (owned)
    // callback
    fosi_hvp_fn fn = nullptr;
    void* user = nullptr;
};

namespace fosi {

// ---- error / profiling helpers (fosi_api.hip) ----
fosi_status fail(fosi_ctx* ctx, fosi_status code, const std::string& msg);
fosi_status check_hip(fosi_ctx* ctx, hipError_t e, const char* what);
void prof_begin(fosi_ctx* ctx, int cls, double bytes);
void prof_end(fosi_ctx* ctx);

struct ProfScope {
    fosi_ctx* c;
    ProfScope(fosi_ctx* ctx, int cls, double bytes) : c(ctx) { prof_begin(c, cls, bytes); }
    ~ProfScope() { prof_end(c); }
};

// ---- kernel launchers (fosi_kernels.hip); all enqueue on ctx->stream ----

// coef[j] = (sum_rows A[row,j] * (x[row] + x2[row])) * (scale ? scale[j] : 1) * gscale  for j < ncols,
// coef[ncols] = sum_rows (x + x2)^2.   x2 and scale may be null.  stop may be null.
// The vector is x, or x + xs[0] x2 (+ xs[1] x3) with xs in device memory (xs == null: scales 1).
// add_last2 (device, may be null): values added to the last and the last-but-one coefficient.
// tail_kind: what the second stage's last workgroup does once all coefficients are in memory, in the same launch:
//   kTailNone;  kTailLocal: ctx->s.loc = {coef[ncols-1], ncols > 1 ? coef[0] : 0, coef[ncols]} and their negatives
//   in ctx->s.scal[4..5] (transposed product against [q_{i-1}, q_i] or [q_i]);  kTailLanczosStep: end of step
//   tail_step of a 'local_full' run (alpha, beta, flags and 1/beta from the coefficients and ctx->s.loc, before
//   the subtraction sweep; same arithmetic as launch_lanczos_finalize_early);  kTailSelectFirst / kTailSelectSecond:
//   the two passes of the 'selective' scheme (the first decides, with ctx->reorth_eta, whether it ends the step
//   or ctx->s.flags[3] lets the second pass's kernels run).
constexpr int kTailNone = 0, kTailLocal = 1, kTailLanczosStep = 2, kTailSelectFirst = 3, kTailSelectSecond = 4;
void launch_dot_columns(fosi_ctx* ctx, const float* A, int64_t lda, int ncols, const float* x,
                        const float* x2, const float* x3, const double* xs, int64_t n, double* coef,
                        const float* scale, int nscale, double gscale, const double* add_last2,
                        const int* stop, int prof_cls, double prof_bytes, int tail_kind = kTailNone,
                        int tail_step = 0, double tail_tol = 0.0);

// out = a0*y + a1*x1 + a2*x2 + sa * A[:, :ncols] d   (null pointers drop their term; out may alias y).
// With want_norm the per-block partial sums of out^2 are left in ctx->s.norm_partials; their count is
// returned.  Only the main kernel of each launcher is bracketed by the profiling events (prof_cls < 0: none).
int launch_combine_columns(fosi_ctx* ctx, const float* A, int64_t lda, int ncols, const double* d,
                           const float* y, double a0, const float* x1, double a1, const float* x2,
                           double a2, const float* x3, bool local_dots, double sa, float* out, int64_t n,
                           bool want_norm, const int* stop, int prof_cls, double prof_bytes,
                           const double* oscale = nullptr);   // oscale (device): factor on the whole result

// cols_a / cols_b: number of columns of the first / second Gram-Schmidt pass (cols_b == 0: single pass);
// in both the current Lanczos vector is the last column of the range.
// 'local_full' scheme: alpha, beta, flags and 1/beta from the full pass's coefficients (coef[cols] = squared norm of
// the vector it worked on) and ctx->s.loc, before the subtraction sweep.
void launch_lanczos_finalize_early(fosi_ctx* ctx, int step, const double* coef, int cols, double tol);
// norm_parts == null: the partial sums the last column-combination kernel left in ctx->s.norm_partials.
void launch_lanczos_finalize(fosi_ctx* ctx, int step, int norm_slots, const double* coef_a, int cols_a,
                             const double* coef_b, int cols_b, const double* hh, double tol,
                             const double* norm_parts = nullptr);
// local_dots variant of launch_combine_columns leaves {out^2, out.x1, out.x3} partials (3 per block);
// this sums them into ctx->s.loc = {alpha~, beta~, ||h||^2} and ctx->s.scal[4..5] = {-alpha~, -beta~}.
void launch_reduce_local(fosi_ctx* ctx, int nslots, const int* stop, const double* parts = nullptr);
// Row-sharded emulation: dst[0..width) = sums over the nslots x width partials in ctx->s.norm_partials.
void launch_fold_partials(fosi_ctx* ctx, int nslots, int width, double* dst, const int* stop);
// ... and the sum over shards of the coefficient rows in ctx->s.xchg (the emulated all-reduce), with the
// post-processing of launch_dot_columns (per-column scale, gscale, add_last2).
void launch_reduce_shards(fosi_ctx* ctx, int shards, int ncols, double* coef, const float* scale, int nscale,
                          double gscale, const double* add_last2, const int* stop);
void launch_local_from_coef(fosi_ctx* ctx, const double* coef, int nc, const int* stop);
void launch_inv_sqrt(fosi_ctx* ctx, const double* in, double* out);
void launch_scale(fosi_ctx* ctx, float* x, const double* factor, int64_t n, const int* stop);
void launch_diag_apply(fosi_ctx* ctx, const float* d, const float* v, float* out, int64_t n);
void launch_ritz_vectors(fosi_ctx* ctx, const float* Q, int64_t ldq, int m, const float* S_dev, int rv_pad,
                         int rv, float* V, int64_t ldv, int64_t n);
// matrix-core variant, 16-wide column blocks, rv <= 64; S_dev is m x (16 ceil(rv / 16)) row-major, zero padded
void launch_traffic_model(fosi_ctx* ctx, const float* A, int64_t lda, int cols_in, float* Bm, int64_t ldb, int cols_out,
                          int64_t n, bool large_tiles);
void launch_ritz_vectors_mfma(fosi_ctx* ctx, const float* Q, int64_t ldq, int m, const float* S_dev, int rv, float* V,
                              int64_t ldv, int64_t n);
void launch_step_coefficients(fosi_ctx* ctx, int rv, double lr);
// Second sweep of the update fused with the transposed product of its result: x = g (+ pi) - V c, base optimiser
// (opt 0: heavy ball on m with factor mu; opt 1: AdamW on m, v with decay against w, descent vector to o_out),
// e_out[j] = sum_rows V[row, j] z[row] with z the new momentum (opt 0) or the descent vector (opt 1).
void launch_complement_reproject(fosi_ctx* ctx, int opt, const float* V, int64_t ldv, int rv, const double* c,
                                 const float* g, const float* pi, const float* w, float* m, float* v, float* o_out,
                                 int64_t n, double mu, double b1, double b2, double inv_bc1, double inv_bc2, double eps,
                                 double lr, double wd, double* e_out, int prof_cls = -1, double prof_bytes = 0.0);
// d = newton . c + e for the last sweep of the AdamW variant
void launch_step_coefficients_plus(fosi_ctx* ctx, int rv);
void launch_admm_begin(fosi_ctx* ctx, int64_t n, double inv_sigma, const float* pi, float* anchor, float* wa);
void launch_admm_end(fosi_ctx* ctx, int64_t n, double sigma, const float* anchor, const float* wa, float* pi);

// softmax-GGN operator (hvp_ggn.hip)
fosi_status ggn_prepare(fosi_hvp* op);
fosi_status ggn_apply(fosi_hvp* op, const float* v, float* hv);
void ggn_release(fosi_hvp* op);

// host tridiagonal eigen-solver (tridiag_eigh.cpp); returns 0 on success
int tridiag_eigh(int m, const double* alpha, const double* beta, double* evals, double* evecs);

}  // namespace fosi
