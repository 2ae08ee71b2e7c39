// The exported C functions: argument checks, the Lanczos driver loop, the host
// part of the Ritz extraction, the sequencing of the update-rule kernels, and
// the opt-in per-kernel timers.  All arithmetic on vectors of length n happens
// in the kernels of fosi_kernels.hip / hvp_ggn.hip.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "fosi_internal.h"

namespace fosi {

fosi_status fail(fosi_ctx* ctx, fosi_status code, const std::string& msg) {
    if (ctx != nullptr) ctx->last_error = msg;
    return code;
}

fosi_status check_hip(fosi_ctx* ctx, hipError_t e, const char* what) {
    if (e == hipSuccess) return FOSI_OK;
    return fail(ctx, FOSI_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

void prof_begin(fosi_ctx* ctx, int cls, double bytes) {
    ctx->prof_open = false;
    if (!ctx->prof_on) return;
    if (ctx->prof_mask != 1 && ((ctx->prof_mask >> (cls + 1)) & 1) == 0) return;   // class not selected
    ProfRecord r{};
    r.cls = cls;
    r.bytes = bytes;
    for (hipEvent_t* ev : {&r.start, &r.stop}) {
        if (!ctx->event_pool.empty()) {
            *ev = ctx->event_pool.back();
            ctx->event_pool.pop_back();
        } else if (hipEventCreate(ev) != hipSuccess) {
            return;
        }
    }
    (void)hipEventRecord(r.start, ctx->stream);
    ctx->prof.push_back(r);
    ctx->prof_open = true;
}

void prof_end(fosi_ctx* ctx) {
    if (!ctx->prof_on || !ctx->prof_open || ctx->prof.empty()) return;
    (void)hipEventRecord(ctx->prof.back().stop, ctx->stream);
    ctx->prof_open = false;
}

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

fosi_status check_matrix(fosi_ctx* ctx, const char* name, const void* p, int64_t n, int64_t ld, int cols) {
    if (cols == 0) return FOSI_OK;
    if (p == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, std::string(name) + " is null");
    if (ld < n || (ld & 3) != 0)
        return fail(ctx, FOSI_ERR_BAD_LAYOUT, std::string(name) + ": leading dimension must be >= n and a multiple of 4");
    if (!aligned16(p)) return fail(ctx, FOSI_ERR_BAD_LAYOUT, std::string(name) + " is not 16-byte aligned");
    return FOSI_OK;
}

fosi_status check_vector(fosi_ctx* ctx, const char* name, const void* p, bool nullable = false) {
    if (p == nullptr) return nullable ? FOSI_OK : fail(ctx, FOSI_ERR_INVALID_ARG, std::string(name) + " is null");
    if (!aligned16(p)) return fail(ctx, FOSI_ERR_BAD_LAYOUT, std::string(name) + " is not 16-byte aligned");
    return FOSI_OK;
}

int env_int(const char* name, int dflt) {
    const char* v = std::getenv(name);
    if (v == nullptr || *v == 0) return dflt;
    return std::atoi(v);
}

size_t round256(size_t b) { return (b + 255) / 256 * 256; }

fosi_status launch_status(fosi_ctx* ctx, const char* what) { return check_hip(ctx, hipGetLastError(), what); }

const double kVec = 4.0;   // bytes per element of an fp32 vector

// Nothing may throw across the C boundary: host allocations (std::vector, std::string) are the only throwing code
// in the library, so every exported function that reaches one runs its body through this.
template <class F>
fosi_status guarded(fosi_ctx* ctx, F&& body) {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        if (ctx != nullptr) {
            try { ctx->last_error = "host allocation failed"; } catch (...) {}
        }
        return FOSI_ERR_NOMEM;
    } catch (...) {
        return FOSI_ERR_INVALID_ARG;
    }
}

// Waits (only) for the previous asynchronous copy out of a pinned staging buffer, if one is still in flight.
fosi_status stage_acquire(fosi_ctx* ctx, hipEvent_t ev, bool& busy) {
    if (!busy) return FOSI_OK;
    busy = false;
    return check_hip(ctx, hipEventSynchronize(ev), "staging buffer");
}

}  // namespace
}  // namespace fosi

using namespace fosi;

extern "C" {

const char* fosi_status_string(fosi_status s) {
    switch (s) {
        case FOSI_OK: return "ok";
        case FOSI_ERR_INVALID_ARG: return "invalid argument";
        case FOSI_ERR_BAD_LAYOUT: return "bad layout";
        case FOSI_ERR_RANK: return "not enough Lanczos steps for the requested Ritz pairs";
        case FOSI_ERR_NONFINITE: return "non-finite value";
        case FOSI_ERR_HIP: return "HIP runtime error";
        case FOSI_ERR_NOMEM: return "out of memory";
        case FOSI_ERR_CALLBACK: return "hvp callback failed";
        case FOSI_ERR_LIMIT: return "size exceeds a built-in limit";
        default: return "unknown status";
    }
}

fosi_status fosi_ctx_create(fosi_ctx** out, int device, void* hip_stream) {
    if (out == nullptr) return FOSI_ERR_INVALID_ARG;
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return FOSI_ERR_HIP;
    if (device < 0 || device >= ndev) return FOSI_ERR_INVALID_ARG;
    if (hipSetDevice(device) != hipSuccess) return FOSI_ERR_HIP;
    fosi_ctx* ctx = new (std::nothrow) fosi_ctx();
    if (ctx == nullptr) return FOSI_ERR_NOMEM;
    ctx->device = device;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) == hipSuccess) ctx->sm_count = prop.multiProcessorCount;
    ctx->tun.dot_target_blocks = env_int("FOSI_DOT_BLOCKS", 0);       // 0: chosen by size
    ctx->tun.dot_slot_cols = env_int("FOSI_DOT_JB", 0);
    ctx->tun.comb_rows_per_thread = env_int("FOSI_COMB_ROWS", 0);   // 0: chosen by size
    ctx->tun.comb_cols_unroll = env_int("FOSI_COMB_COLS", 0);
    ctx->tun.comb_max_blocks = env_int("FOSI_COMB_BLOCKS", 0);
    ctx->tun.early_beta = env_int("FOSI_EARLY_BETA", 1);
    ctx->tun.ritz_mfma = env_int("FOSI_RITZ_MFMA", 1);
    ctx->tun.step_waves_per_cu = env_int("FOSI_STEP_WAVES", 8);
    ctx->tun.step_cols_per_wave = env_int("FOSI_STEP_COLS", 0);
    ctx->tun.ggn_direct = env_int("FOSI_GGN_DIRECT", 1);
    if (ctx->tun.step_waves_per_cu < 1) ctx->tun.step_waves_per_cu = 1;

    const size_t cols1 = kMaxCols + 1;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += round256(bytes); return o; };
    const size_t o_part = take(sizeof(double) * kMaxDotSlots * cols1);
    const size_t o_norm = take(sizeof(double) * 3 * kMaxNormSlots);
    const size_t o_ca = take(sizeof(double) * cols1), o_cb = take(sizeof(double) * cols1);
    const size_t o_cc = take(sizeof(double) * cols1), o_ch = take(sizeof(double) * cols1);
    const size_t o_scal = take(sizeof(double) * 8);
    const size_t o_loc = take(sizeof(double) * 8);
    const size_t o_al = take(sizeof(double) * kMaxCols), o_be = take(sizeof(double) * kMaxCols);
    const size_t o_hn = take(sizeof(double) * kMaxCols), o_nw = take(sizeof(double) * kMaxCols);
    const size_t o_S = take(sizeof(float) * kMaxCols * kMaxCols);
    const size_t o_fl = take(sizeof(int) * 8);
    const size_t o_x = take(sizeof(double) * kMaxShards * cols1), o_x3 = take(sizeof(double) * kMaxShards * 3);
    ctx->scratch_bytes = off;
    if (hipMalloc(&ctx->scratch_base, off) != hipSuccess) {
        delete ctx;
        return FOSI_ERR_NOMEM;
    }
    if (hipHostMalloc(reinterpret_cast<void**>(&ctx->stage_S), sizeof(float) * kMaxCols * 64, hipHostMallocDefault) != hipSuccess ||
        hipHostMalloc(reinterpret_cast<void**>(&ctx->stage_newton), sizeof(double) * kMaxCols, hipHostMallocDefault) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->stage_S_done, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&ctx->stage_newton_done, hipEventDisableTiming) != hipSuccess) {
        if (ctx->stage_S != nullptr) (void)hipHostFree(ctx->stage_S);
        if (ctx->stage_newton != nullptr) (void)hipHostFree(ctx->stage_newton);
        if (ctx->stage_S_done != nullptr) (void)hipEventDestroy(ctx->stage_S_done);
        if (ctx->stage_newton_done != nullptr) (void)hipEventDestroy(ctx->stage_newton_done);
        (void)hipFree(ctx->scratch_base);
        delete ctx;
        return FOSI_ERR_NOMEM;
    }
    char* b = static_cast<char*>(ctx->scratch_base);
    ctx->s.partials = reinterpret_cast<double*>(b + o_part);
    ctx->s.norm_partials = reinterpret_cast<double*>(b + o_norm);
    ctx->s.coef_a = reinterpret_cast<double*>(b + o_ca);
    ctx->s.coef_b = reinterpret_cast<double*>(b + o_cb);
    ctx->s.coef_c = reinterpret_cast<double*>(b + o_cc);
    ctx->s.coef_h = reinterpret_cast<double*>(b + o_ch);
    ctx->s.scal = reinterpret_cast<double*>(b + o_scal);
    ctx->s.loc = reinterpret_cast<double*>(b + o_loc);
    ctx->s.alpha = reinterpret_cast<double*>(b + o_al);
    ctx->s.beta = reinterpret_cast<double*>(b + o_be);
    ctx->s.hnorm = reinterpret_cast<double*>(b + o_hn);
    ctx->s.newton = reinterpret_cast<double*>(b + o_nw);
    ctx->s.S = reinterpret_cast<float*>(b + o_S);
    ctx->s.flags = reinterpret_cast<int*>(b + o_fl);
    ctx->s.xchg = reinterpret_cast<double*>(b + o_x);
    ctx->s.xchg3 = reinterpret_cast<double*>(b + o_x3);
    const double ones[2] = {1.0, 1.0};
    if (hipMemsetAsync(ctx->scratch_base, 0, off, ctx->stream) != hipSuccess ||
        hipMemcpyAsync(ctx->s.scal + 2, ones, sizeof(ones), hipMemcpyHostToDevice, ctx->stream) != hipSuccess ||
        hipStreamSynchronize(ctx->stream) != hipSuccess) {
        (void)hipHostFree(ctx->stage_S);
        (void)hipHostFree(ctx->stage_newton);
        (void)hipEventDestroy(ctx->stage_S_done);
        (void)hipEventDestroy(ctx->stage_newton_done);
        (void)hipFree(ctx->scratch_base);
        delete ctx;
        return FOSI_ERR_HIP;
    }
    *out = ctx;
    return FOSI_OK;
}

fosi_status fosi_ctx_destroy(fosi_ctx* ctx) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    (void)hipStreamSynchronize(ctx->stream);
    for (auto& r : ctx->prof) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    for (auto& e : ctx->event_pool) (void)hipEventDestroy(e);
    if (ctx->graph_exec != nullptr) (void)hipGraphExecDestroy(ctx->graph_exec);
    (void)hipHostFree(ctx->stage_S);
    (void)hipHostFree(ctx->stage_newton);
    (void)hipEventDestroy(ctx->stage_S_done);
    (void)hipEventDestroy(ctx->stage_newton_done);
    (void)hipFree(ctx->scratch_base);
    delete ctx;
    return FOSI_OK;
}

size_t fosi_workspace_bytes(int64_t n, int m, int r_v) {
    if (n < 1 || m < 1 || r_v < 0 || m + 1 > kMaxCols || r_v > kMaxCols) return 0;
    // the same layout fosi_ctx_create allocates: sized by the built-in limits, not by (n, m, r_v)
    const size_t cols1 = kMaxCols + 1;
    size_t off = 0;
    auto take = [&](size_t bytes) { off += round256(bytes); };
    take(sizeof(double) * kMaxDotSlots * cols1);
    take(sizeof(double) * 3 * kMaxNormSlots);
    for (int i = 0; i < 4; ++i) take(sizeof(double) * cols1);
    take(sizeof(double) * 8);
    take(sizeof(double) * 8);
    for (int i = 0; i < 4; ++i) take(sizeof(double) * kMaxCols);
    take(sizeof(float) * kMaxCols * kMaxCols);
    take(sizeof(int) * 8);
    take(sizeof(double) * kMaxShards * cols1);
    take(sizeof(double) * kMaxShards * 3);
    return off;
}

fosi_status fosi_ctx_synchronize(fosi_ctx* ctx) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    return check_hip(ctx, hipStreamSynchronize(ctx->stream), "hipStreamSynchronize");
}

const char* fosi_last_error(const fosi_ctx* ctx) { return ctx == nullptr ? "null context" : ctx->last_error.c_str(); }

/* ------------------------------------------------------------- operators */

static fosi_status new_op(fosi_ctx* ctx, fosi_hvp::Kind kind, int64_t n, fosi_hvp** out) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (out == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (n < 1) return fail(ctx, FOSI_ERR_INVALID_ARG, "n must be positive");
    fosi_hvp* op = new (std::nothrow) fosi_hvp();
    if (op == nullptr) return fail(ctx, FOSI_ERR_NOMEM, "operator allocation failed");
    op->kind = kind;
    op->ctx = ctx;
    op->n = n;
    *out = op;
    return FOSI_OK;
}

static fosi_status hvp_planted_create_impl(fosi_ctx* ctx, int64_t n, int r, const float* U_dev, int64_t ldu,
                               const float* lam_dev, float shift, fosi_hvp** out) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (out != nullptr) *out = nullptr;
    if (n < 1 || r < 0) return fail(ctx, FOSI_ERR_INVALID_ARG, "n must be positive and r non-negative");
    if (r > kMaxCols) return fail(ctx, FOSI_ERR_LIMIT, "planted rank exceeds FOSI_MAX_COLS");
    if (fosi_status s = check_matrix(ctx, "U_dev", U_dev, n, ldu, r)) return s;
    if (r > 0 && lam_dev == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, "lam_dev is null");
    if (fosi_status s = new_op(ctx, fosi_hvp::PLANTED, n, out)) return s;
    (*out)->r = r;
    (*out)->U = U_dev;
    (*out)->ldu = ldu;
    (*out)->lam = lam_dev;
    (*out)->shift = shift;
    return FOSI_OK;
}

static fosi_status hvp_diag_create_impl(fosi_ctx* ctx, int64_t n, const float* d_dev, fosi_hvp** out) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (out != nullptr) *out = nullptr;
    if (d_dev == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, "d_dev is null");
    if (fosi_status s = new_op(ctx, fosi_hvp::DIAG, n, out)) return s;
    (*out)->d = d_dev;
    return FOSI_OK;
}

static fosi_status hvp_softmax_ggn_create_impl(fosi_ctx* ctx, int B, int d, int C, const float* X_dev, const float* W_dev,
                                   fosi_hvp** out) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (out != nullptr) *out = nullptr;
    if (B < 1 || d < 1 || C < 1) return fail(ctx, FOSI_ERR_INVALID_ARG, "B, d, C must be positive");
    if (X_dev == nullptr || W_dev == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, "X_dev or W_dev is null");
    if (!aligned16(X_dev) || !aligned16(W_dev)) return fail(ctx, FOSI_ERR_BAD_LAYOUT, "X_dev/W_dev not 16-byte aligned");
    if (fosi_status s = new_op(ctx, fosi_hvp::GGN, (int64_t)d * C, out)) return s;
    fosi_hvp* op = *out;
    op->B = B;
    op->dim = d;
    op->C = C;
    op->X = X_dev;
    op->W = W_dev;
    if (fosi_status s = ggn_prepare(op)) {
        ggn_release(op);
        delete op;
        *out = nullptr;
        return s;
    }
    return FOSI_OK;
}

static fosi_status hvp_softmax_ggn_bf16_create_impl(fosi_ctx* ctx, int B, int d, int C, const uint16_t* X_bf16_dev,
                                        const float* W_dev, fosi_hvp** out) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (out != nullptr) *out = nullptr;
    if (B < 1 || d < 1 || C < 1) return fail(ctx, FOSI_ERR_INVALID_ARG, "B, d, C must be positive");
    if (X_bf16_dev == nullptr || W_dev == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, "X_bf16_dev or W_dev is null");
    if (!aligned16(X_bf16_dev) || !aligned16(W_dev))
        return fail(ctx, FOSI_ERR_BAD_LAYOUT, "X_bf16_dev/W_dev not 16-byte aligned");
    if (fosi_status s = new_op(ctx, fosi_hvp::GGN, (int64_t)d * C, out)) return s;
    fosi_hvp* op = *out;
    op->B = B;
    op->dim = d;
    op->C = C;
    op->bf16 = true;
    op->Xb = X_bf16_dev;
    op->W = W_dev;
    if (fosi_status s = ggn_prepare(op)) {
        ggn_release(op);
        delete op;
        *out = nullptr;
        return s;
    }
    return FOSI_OK;
}

static fosi_status hvp_callback_create_impl(fosi_ctx* ctx, int64_t n, fosi_hvp_fn fn, void* user, fosi_hvp** out) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (out != nullptr) *out = nullptr;
    if (fn == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, "fn is null");
    if (fosi_status s = new_op(ctx, fosi_hvp::CALLBACK, n, out)) return s;
    (*out)->fn = fn;
    (*out)->user = user;
    return FOSI_OK;
}

// Applies the operator.  With want_local the scalars of the local Gram-Schmidt pass are produced as
// well: ctx->s.loc = {hv . v, hv . vprev, ||hv||^2} (vprev may be null: second entry 0) and their
// negatives in ctx->s.scal[4..5].  The planted operator gets them for free inside its expand sweep;
// the other operators pay one transposed product against [vprev, v].
static fosi_status apply_operator(fosi_hvp* op, const float* v_dev, float* hv_dev, const float* vprev,
                                  bool want_local) {
    fosi_ctx* ctx = op->ctx;
    const int64_t n = op->n;
    const int* stop = ctx->s.flags;   // zero outside a Lanczos run
    const double vec = kVec * (double)n;
    switch (op->kind) {
        case fosi_hvp::PLANTED: {
            // coefficients lam_j * (u_j . v), then shift v + U (coefficients)
            launch_dot_columns(ctx, op->U, op->ldu, op->r, v_dev, nullptr, nullptr, nullptr, n, ctx->s.coef_h, op->lam,
                               op->r, 1.0, nullptr, stop, FOSI_PROF_HVP_PROJECT, (op->r + 1) * vec);
            const int extra = (want_local && vprev != nullptr) ? 1 : 0;
            const int slots = launch_combine_columns(ctx, op->U, op->ldu, op->r, ctx->s.coef_h, nullptr, 0.0, v_dev,
                                                     (double)op->shift, nullptr, 0.0, vprev, want_local, 1.0, hv_dev, n,
                                                     false, stop, FOSI_PROF_HVP_EXPAND, (op->r + 2 + extra) * vec);
            if (want_local) launch_reduce_local(ctx, slots, stop);
            return launch_status(ctx, "hvp_apply");
        }
        case fosi_hvp::DIAG: {
            ProfScope p(ctx, FOSI_PROF_HVP_OTHER, 3 * vec);
            launch_diag_apply(ctx, op->d, v_dev, hv_dev, n);
            break;
        }
        case fosi_hvp::GGN: {
            // for this class the "bytes" slot carries the floating-point operations of the two GEMMs
            ProfScope p(ctx, FOSI_PROF_HVP_GGN, 4.0 * op->B * (double)op->dim * op->C);
            if (fosi_status s = ggn_apply(op, v_dev, hv_dev)) return s;
            break;
        }
        case fosi_hvp::CALLBACK: {
            ProfScope p(ctx, FOSI_PROF_HVP_OTHER, 0.0);
            if (op->fn(op->user, v_dev, hv_dev, ctx->stream) != 0)
                return fail(ctx, FOSI_ERR_CALLBACK, "hvp callback returned non-zero");
            break;
        }
    }
    if (want_local) {
        // vprev, when given, is the column just before v in the caller's matrix
        const int nc = vprev != nullptr ? 2 : 1;
        const float* base = vprev != nullptr ? vprev : v_dev;
        const int64_t ld = vprev != nullptr ? (int64_t)(v_dev - vprev) : 0;
        launch_dot_columns(ctx, base, ld, nc, hv_dev, nullptr, nullptr, nullptr, n, ctx->s.coef_a, nullptr, 0, 1.0,
                           nullptr, stop, FOSI_PROF_REORTH_DOT, (nc + 1) * vec, kTailLocal);
    }
    return launch_status(ctx, "hvp_apply");
}

static fosi_status hvp_apply_impl(fosi_hvp* op, const float* v_dev, float* hv_dev) {
    if (op == nullptr) return FOSI_ERR_INVALID_ARG;
    fosi_ctx* ctx = op->ctx;
    if (fosi_status s = check_vector(ctx, "v_dev", v_dev)) return s;
    if (fosi_status s = check_vector(ctx, "hv_dev", hv_dev)) return s;
    if (v_dev == hv_dev) return fail(ctx, FOSI_ERR_INVALID_ARG, "v_dev and hv_dev must be distinct");
    return apply_operator(op, v_dev, hv_dev, nullptr, false);
}

static void drop_graph(fosi_ctx* ctx);

static fosi_status hvp_destroy_impl(fosi_hvp* op) {
    if (op == nullptr) return FOSI_ERR_INVALID_ARG;
    if (op->ctx->graph_key.op == op) {      // a captured run refers to this operator's buffers
        (void)hipStreamSynchronize(op->ctx->stream);
        drop_graph(op->ctx);
    }
    if (op->kind == fosi_hvp::GGN) {
        (void)hipStreamSynchronize(op->ctx->stream);
        ggn_release(op);
    }
    delete op;
    return FOSI_OK;
}

/* ------------------------------------------------------------- Algorithm 1 */

int32_t fosi_lanczos_steps(int64_t n, int k, int l) {
    if (n < 1 || k < 0 || l < 0 || k + l < 1) return 0;
    const double by_pairs = 4.0 * (k + l), by_size = 2.0 * std::log((double)n);
    return (int32_t)std::ceil(by_pairs > by_size ? by_pairs : by_size);
}

// Enqueues the start-vector normalisation and the m steps of Algorithm 1 on the context's stream; nothing
// here waits for the device, so the same sequence can be recorded into a graph.
static fosi_status enqueue_lanczos(fosi_ctx* ctx, fosi_hvp* op, int64_t n, int m, float* Q_dev, int64_t ldq, int mode,
                                   double tol) {
    const int passes = mode == FOSI_REORTH_SINGLE ? 1 : 2;
    const double vec = kVec * (double)n;
    int* flags = ctx->s.flags;
    // first column: the caller's vector, normalised in place
    launch_dot_columns(ctx, nullptr, 0, 0, Q_dev, nullptr, nullptr, nullptr, n, ctx->s.coef_a, nullptr, 0, 1.0, nullptr,
                       nullptr, -1, 0.0);
    launch_inv_sqrt(ctx, ctx->s.coef_a, ctx->s.scal + 1);
    launch_scale(ctx, Q_dev, ctx->s.scal + 1, n, nullptr);

    for (int i = 0; i < m; ++i) {
        const float* q = Q_dev + (int64_t)i * ldq;
        float* h = Q_dev + (int64_t)(i + 1) * ldq;     // the new direction is built in place in the next column
        const int ncols = i + 1;
        int norm_slots = 0;
        if (mode == FOSI_REORTH_LOCAL_FULL) {
            // local pass: alpha~ = h . q_i and beta~ = h . q_{i-1} come with the operator; h itself is left
            // untouched and the full pass works on h - alpha~ q_i - beta~ q_{i-1}, formed on the fly in fp64
            const float* qprev = i > 0 ? q - ldq : nullptr;
            if (fosi_status s = apply_operator(op, q, h, qprev, true)) return s;
            // coef_b receives the total coefficient per column (local + full); one subtraction removes both
            if (ctx->tun.early_beta) {
                // beta from the coefficients (by the last workgroup of the product's second stage), then the
                // subtraction writes the normalised vector itself
                launch_dot_columns(ctx, Q_dev, ldq, ncols, h, q, qprev, ctx->s.scal + 4, n, ctx->s.coef_b, nullptr, 0, 1.0,
                                   ctx->s.loc, flags, FOSI_PROF_REORTH_DOT, (ncols + 1 + (qprev != nullptr ? 2 : 1)) * vec,
                                   kTailLanczosStep, i, tol);
                launch_combine_columns(ctx, Q_dev, ldq, ncols, ctx->s.coef_b, h, 1.0, nullptr, 0.0, nullptr, 0.0, nullptr,
                                       false, -1.0, h, n, false, flags, FOSI_PROF_REORTH_SUB, (ncols + 2) * vec,
                                       ctx->s.scal);
                if (fosi_status s = launch_status(ctx, "lanczos step")) return s;
                continue;
            }
            launch_dot_columns(ctx, Q_dev, ldq, ncols, h, q, qprev, ctx->s.scal + 4, n, ctx->s.coef_b, nullptr, 0, 1.0,
                               ctx->s.loc, flags, FOSI_PROF_REORTH_DOT, (ncols + 1 + (qprev != nullptr ? 2 : 1)) * vec);
            norm_slots = launch_combine_columns(ctx, Q_dev, ldq, ncols, ctx->s.coef_b, h, 1.0, nullptr, 0.0, nullptr,
                                                0.0, nullptr, false, -1.0, h, n, true, flags, FOSI_PROF_REORTH_SUB,
                                                (ncols + 2) * vec);
            launch_lanczos_finalize(ctx, i, norm_slots, ctx->s.coef_b, ncols, nullptr, 0, ctx->s.loc + 2, tol);
        } else if (mode == FOSI_REORTH_SELECTIVE) {
            if (fosi_status s = apply_operator(op, q, h, nullptr, false)) return s;
            // first pass; the last workgroup of its second stage either ends the step (beta from the
            // coefficients, the subtraction writes the normalised vector) or, when much was cancelled, leaves
            // the subtraction unscaled and clears flags[3], on which the kernels of the second pass wait
            launch_dot_columns(ctx, Q_dev, ldq, ncols, h, nullptr, nullptr, nullptr, n, ctx->s.coef_a, nullptr, 0, 1.0,
                               nullptr, flags, FOSI_PROF_REORTH_DOT, (ncols + 1) * vec, kTailSelectFirst, i, tol);
            launch_combine_columns(ctx, Q_dev, ldq, ncols, ctx->s.coef_a, h, 1.0, nullptr, 0.0, nullptr, 0.0, nullptr,
                                   false, -1.0, h, n, false, flags, FOSI_PROF_REORTH_SUB, (ncols + 2) * vec, ctx->s.scal);
            launch_dot_columns(ctx, Q_dev, ldq, ncols, h, nullptr, nullptr, nullptr, n, ctx->s.coef_b, nullptr, 0, 1.0,
                               nullptr, flags + 3, FOSI_PROF_REORTH_DOT, (ncols + 1) * vec, kTailSelectSecond, i, tol);
            launch_combine_columns(ctx, Q_dev, ldq, ncols, ctx->s.coef_b, h, 1.0, nullptr, 0.0, nullptr, 0.0, nullptr,
                                   false, -1.0, h, n, false, flags + 3, FOSI_PROF_REORTH_SUB, (ncols + 2) * vec,
                                   ctx->s.scal);
            if (fosi_status s = launch_status(ctx, "lanczos step")) return s;
            continue;
        } else {
            if (fosi_status s = apply_operator(op, q, h, nullptr, false)) return s;
            double* coef[2] = {ctx->s.coef_a, ctx->s.coef_b};
            for (int p = 0; p < passes; ++p) {
                // Gram-Schmidt against every column built so far; the coefficient along q_i is the diagonal entry
                launch_dot_columns(ctx, Q_dev, ldq, ncols, h, nullptr, nullptr, nullptr, n, coef[p], nullptr, 0, 1.0,
                                   nullptr, flags, FOSI_PROF_REORTH_DOT, (ncols + 1) * vec);
                norm_slots = launch_combine_columns(ctx, Q_dev, ldq, ncols, coef[p], h, 1.0, nullptr, 0.0, nullptr, 0.0,
                                                    nullptr, false, -1.0, h, n, true, flags, FOSI_PROF_REORTH_SUB,
                                                    (ncols + 2) * vec);
            }
            launch_lanczos_finalize(ctx, i, norm_slots, ctx->s.coef_a, ncols, passes == 2 ? ctx->s.coef_b : nullptr,
                                    passes == 2 ? ncols : 0, nullptr, tol);
        }
        {
            ProfScope ps(ctx, FOSI_PROF_NORMALISE, 2 * vec);
            launch_scale(ctx, h, ctx->s.scal, n, flags);
        }
        if (fosi_status s = launch_status(ctx, "lanczos step")) return s;
    }
    return FOSI_OK;
}

static void drop_graph(fosi_ctx* ctx) {
    if (ctx->graph_exec != nullptr) (void)hipGraphExecDestroy(ctx->graph_exec);
    ctx->graph_exec = nullptr;
    ctx->graph_key = fosi_ctx::GraphKey{};
}

// Replays the cached graph of this run, capturing it first when the key differs.  Returns false when the
// stream cannot be captured (the caller then launches eagerly); *st carries an error from the enqueue itself.
static bool lanczos_by_graph(fosi_ctx* ctx, fosi_hvp* op, int64_t n, int m, float* Q_dev, int64_t ldq, int mode,
                             double tol, fosi_status* st) {
    *st = FOSI_OK;
    fosi_ctx::GraphKey key;
    key.op = op; key.Q = Q_dev; key.n = n; key.ldq = ldq; key.m = m; key.mode = mode; key.tol = tol;
    key.eta = ctx->reorth_eta;
    if (ctx->graph_exec == nullptr || !(ctx->graph_key == key)) {
        drop_graph(ctx);
        if (hipStreamBeginCapture(ctx->stream, hipStreamCaptureModeRelaxed) != hipSuccess) {
            (void)hipGetLastError();
            ctx->graph_unavailable = true;
            return false;
        }
        const fosi_status es = enqueue_lanczos(ctx, op, n, m, Q_dev, ldq, mode, tol);
        hipGraph_t graph = nullptr;
        const hipError_t ee = hipStreamEndCapture(ctx->stream, &graph);
        if (es != FOSI_OK || ee != hipSuccess || graph == nullptr) {
            if (graph != nullptr) (void)hipGraphDestroy(graph);
            (void)hipGetLastError();
            if (es != FOSI_OK) { *st = es; return true; }
            ctx->graph_unavailable = true;
            return false;
        }
        const hipError_t ie = hipGraphInstantiate(&ctx->graph_exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (ie != hipSuccess) {
            (void)hipGetLastError();
            ctx->graph_exec = nullptr;
            ctx->graph_unavailable = true;
            return false;
        }
        ctx->graph_key = key;
        ++ctx->graph_captures;
    }
    *st = check_hip(ctx, hipGraphLaunch(ctx->graph_exec, ctx->stream), "hipGraphLaunch");
    if (*st == FOSI_OK) ++ctx->graph_replays;
    return true;
}

static fosi_status fosi_lanczos_begin_impl(fosi_ctx* ctx, fosi_hvp* op, int64_t n, int m, float* Q_dev, int64_t ldq,
                               const fosi_lanczos_opts* opts) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (op == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, "null argument");
    if (op->ctx != ctx) return fail(ctx, FOSI_ERR_INVALID_ARG, "operator belongs to another context");
    if (n < 1 || m < 1) return fail(ctx, FOSI_ERR_INVALID_ARG, "n and m must be positive");
    if (op->n != n) return fail(ctx, FOSI_ERR_INVALID_ARG, "operator size differs from n");
    if (m + 1 > kMaxCols) return fail(ctx, FOSI_ERR_LIMIT, "m + 1 exceeds FOSI_MAX_COLS");
    if (ctx->pending_m != 0) return fail(ctx, FOSI_ERR_INVALID_ARG, "a Lanczos run is already pending on this context");
    if (fosi_status s = check_matrix(ctx, "Q_dev", Q_dev, n, ldq, m + 1)) return s;
    int mode = FOSI_REORTH_LOCAL_FULL, graph_mode = FOSI_GRAPH_OFF;
    double tol = 1e-6;
    if (opts != nullptr) {
        if (opts->reorth_mode != 0) mode = opts->reorth_mode;
        if (opts->breakdown_tol > 0.0) tol = opts->breakdown_tol;
        graph_mode = opts->graph_mode;
    }
    if (mode != FOSI_REORTH_SINGLE && mode != FOSI_REORTH_TWICE && mode != FOSI_REORTH_LOCAL_FULL &&
        mode != FOSI_REORTH_SELECTIVE)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "unknown reorth_mode");
    if (graph_mode != FOSI_GRAPH_OFF && graph_mode != FOSI_GRAPH_ON)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "unknown graph_mode");
    double eta = 0.70710678118654752;
    if (opts != nullptr && opts->reorth_eta != 0.0) eta = opts->reorth_eta;
    if (!(eta > 0.0 && eta < 1.0)) return fail(ctx, FOSI_ERR_INVALID_ARG, "reorth_eta must lie in (0, 1)");
    ctx->reorth_eta = eta;

    int* flags = ctx->s.flags;
    // (cleared outside the graph: memset nodes are kept out of captured work)
    if (fosi_status s = check_hip(ctx, hipMemsetAsync(flags, 0, 8 * sizeof(int), ctx->stream), "clear flags")) return s;

    const bool graph_wanted = graph_mode == FOSI_GRAPH_ON && ctx->stream != nullptr && !ctx->graph_unavailable &&
                              !ctx->prof_on && op->kind != fosi_hvp::CALLBACK;
    bool done = false;
    if (graph_wanted) {
        fosi_status gs = FOSI_OK;
        done = lanczos_by_graph(ctx, op, n, m, Q_dev, ldq, mode, tol, &gs);
        if (done && gs != FOSI_OK) return gs;
    }
    if (!done)
        if (fosi_status s = enqueue_lanczos(ctx, op, n, m, Q_dev, ldq, mode, tol)) return s;
    ctx->pending_m = m;
    return FOSI_OK;
}

static fosi_status fosi_lanczos_end_impl(fosi_ctx* ctx, double* alpha_host, double* beta_host, int32_t* m_eff) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (alpha_host == nullptr || beta_host == nullptr || m_eff == nullptr)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "null argument");
    if (ctx->pending_m == 0) return fail(ctx, FOSI_ERR_INVALID_ARG, "no Lanczos run is pending on this context");
    const int m = ctx->pending_m;
    ctx->pending_m = 0;
    *m_eff = 0;
    int* flags = ctx->s.flags;
    int hflags[5] = {0, 0, 0, 0, 0};
    if (fosi_status s = check_hip(ctx, hipMemcpyAsync(alpha_host, ctx->s.alpha, sizeof(double) * m, hipMemcpyDeviceToHost,
                                                      ctx->stream), "copy alpha")) return s;
    if (fosi_status s = check_hip(ctx, hipMemcpyAsync(beta_host, ctx->s.beta, sizeof(double) * m, hipMemcpyDeviceToHost,
                                                      ctx->stream), "copy beta")) return s;
    if (fosi_status s = check_hip(ctx, hipMemcpyAsync(hflags, flags, sizeof(hflags), hipMemcpyDeviceToHost, ctx->stream),
                                  "copy flags")) return s;
    if (fosi_status s = check_hip(ctx, hipStreamSynchronize(ctx->stream), "lanczos synchronize")) return s;
    // leave the stop flag clear so that later operator applications run
    if (fosi_status s = check_hip(ctx, hipMemsetAsync(flags, 0, 8 * sizeof(int), ctx->stream), "clear flags")) return s;
    *m_eff = hflags[1];
    ctx->second_passes = hflags[4];
    if (hflags[0] == 2) return fail(ctx, FOSI_ERR_NONFINITE, "non-finite value in the Lanczos recurrence");
    return FOSI_OK;
}

fosi_status fosi_lanczos(fosi_ctx* ctx, fosi_hvp* op, int64_t n, int m, float* Q_dev, int64_t ldq,
                         double* alpha_host, double* beta_host, int32_t* m_eff, const fosi_lanczos_opts* opts) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (alpha_host == nullptr || beta_host == nullptr || m_eff == nullptr)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "null argument");
    *m_eff = 0;
    if (fosi_status s = fosi_lanczos_begin(ctx, op, n, m, Q_dev, ldq, opts)) return s;
    return fosi_lanczos_end(ctx, alpha_host, beta_host, m_eff);
}

/* Number of graph captures and replays of this context so far (for tests and diagnostics). */
fosi_status fosi_graph_stats(fosi_ctx* ctx, int64_t* captures, int64_t* replays) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (captures != nullptr) *captures = ctx->graph_captures;
    if (replays != nullptr) *replays = ctx->graph_replays;
    return FOSI_OK;
}

fosi_status fosi_lanczos_second_passes(fosi_ctx* ctx, int32_t* count) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (count == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, "null argument");
    *count = ctx->second_passes;
    return FOSI_OK;
}

/* ------------------------------------------------- Algorithm 2 on one GPU */

struct Shards {
    int count = 0;
    int64_t begin[kMaxShards + 1] = {0};
    int64_t rows(int c) const { return begin[c + 1] - begin[c]; }
};

// Contiguous row blocks with boundaries at multiples of 64 rows (so that every block starts 256-byte
// aligned); blocks that would be empty are dropped.
static Shards make_shards(int64_t n, int want) {
    Shards sh;
    const int64_t per = ((n + want - 1) / want + 63) / 64 * 64;
    int64_t s = 0;
    while (s < n && sh.count < want) {
        sh.begin[sh.count] = s;
        s = s + per < n ? s + per : n;
        sh.begin[++sh.count] = s;
    }
    return sh;
}

// c = A^T (x [+ xs0 x2 + xs1 x3]) with the rows cut into blocks: one sweep per block into its row of the
// exchange buffer, then the sum over blocks (where the distributed algorithm has its all-reduce).
static void sharded_dot(fosi_ctx* ctx, const Shards& sh, const float* A, int64_t lda, int ncols, const float* x,
                 const float* x2, const float* x3, const double* xs, double* coef, const float* scale, int nscale,
                 const double* add_last2, const int* stop, int prof_cls) {
    for (int c = 0; c < sh.count; ++c) {
        const int64_t o = sh.begin[c], nr = sh.rows(c);
        const int nx = 1 + (x2 != nullptr) + (x3 != nullptr);
        launch_dot_columns(ctx, A != nullptr ? A + o : nullptr, lda, ncols, x + o, x2 != nullptr ? x2 + o : nullptr,
                           x3 != nullptr ? x3 + o : nullptr, xs, nr, ctx->s.xchg + (size_t)c * (kMaxCols + 1), nullptr, 0,
                           1.0, nullptr, stop, prof_cls, (ncols + nx) * kVec * (double)nr);
    }
    launch_reduce_shards(ctx, sh.count, ncols, coef, scale, nscale, 1.0, add_last2, stop);
}

// h <- h - Q c on every block; the blocks' parts of ||h||^2 go to xchg3[c].
static void sharded_subtract(fosi_ctx* ctx, const Shards& sh, const float* Q, int64_t ldq, int ncols, const double* coef,
                      float* h, const int* stop) {
    for (int c = 0; c < sh.count; ++c) {
        const int64_t o = sh.begin[c], nr = sh.rows(c);
        const int slots = launch_combine_columns(ctx, Q + o, ldq, ncols, coef, h + o, 1.0, nullptr, 0.0, nullptr, 0.0,
                                                 nullptr, false, -1.0, h + o, nr, true, stop, FOSI_PROF_REORTH_SUB,
                                                 (ncols + 2) * kVec * (double)nr);
        launch_fold_partials(ctx, slots, 1, ctx->s.xchg3 + c, stop);
    }
}

static fosi_status sharded_operator(fosi_hvp* op, const Shards& sh, const float* v, float* hv, const float* vprev,
                             bool want_local) {
    fosi_ctx* ctx = op->ctx;
    const int* stop = ctx->s.flags;
    if (op->kind == fosi_hvp::PLANTED) {
        sharded_dot(ctx, sh, op->U, op->ldu, op->r, v, nullptr, nullptr, nullptr, ctx->s.coef_h, op->lam, op->r, nullptr,
                    stop, FOSI_PROF_HVP_PROJECT);
        for (int c = 0; c < sh.count; ++c) {
            const int64_t o = sh.begin[c], nr = sh.rows(c);
            const int extra = (want_local && vprev != nullptr) ? 1 : 0;
            const int slots = launch_combine_columns(ctx, op->U + o, op->ldu, op->r, ctx->s.coef_h, nullptr, 0.0, v + o,
                                                     (double)op->shift, nullptr, 0.0, vprev != nullptr ? vprev + o : nullptr,
                                                     want_local, 1.0, hv + o, nr, false, stop, FOSI_PROF_HVP_EXPAND,
                                                     (op->r + 2 + extra) * kVec * (double)nr);
            if (want_local) launch_fold_partials(ctx, slots, 3, ctx->s.xchg3 + 3 * c, stop);
        }
        if (want_local) launch_reduce_local(ctx, sh.count, stop, ctx->s.xchg3);
        return launch_status(ctx, "sharded hvp");
    }
    // other operators see the whole vector; only the local products are taken block by block
    if (fosi_status s = apply_operator(op, v, hv, nullptr, false)) return s;
    if (want_local) {
        const int nc = vprev != nullptr ? 2 : 1;
        const float* base = vprev != nullptr ? vprev : v;
        const int64_t ld = vprev != nullptr ? (int64_t)(v - vprev) : 0;
        sharded_dot(ctx, sh, base, ld, nc, hv, nullptr, nullptr, nullptr, ctx->s.coef_a, nullptr, 0, nullptr, stop,
                    FOSI_PROF_REORTH_DOT);
        launch_local_from_coef(ctx, ctx->s.coef_a, nc, stop);
    }
    return launch_status(ctx, "sharded hvp");
}

static fosi_status fosi_lanczos_row_sharded_impl(fosi_ctx* ctx, fosi_hvp* op, int64_t n, int m, int shards, float* Q_dev,
                                     int64_t ldq, double* alpha_host, double* beta_host, int32_t* m_eff,
                                     const fosi_lanczos_opts* opts) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (op == nullptr || alpha_host == nullptr || beta_host == nullptr || m_eff == nullptr)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "null argument");
    if (op->ctx != ctx) return fail(ctx, FOSI_ERR_INVALID_ARG, "operator belongs to another context");
    if (n < 1 || m < 1) return fail(ctx, FOSI_ERR_INVALID_ARG, "n and m must be positive");
    if (shards < 1) return fail(ctx, FOSI_ERR_INVALID_ARG, "shards must be positive");
    if (shards > kMaxShards) return fail(ctx, FOSI_ERR_LIMIT, "shards exceeds FOSI_MAX_SHARDS");
    if (op->n != n) return fail(ctx, FOSI_ERR_INVALID_ARG, "operator size differs from n");
    if (m + 1 > kMaxCols) return fail(ctx, FOSI_ERR_LIMIT, "m + 1 exceeds FOSI_MAX_COLS");
    if (fosi_status s = check_matrix(ctx, "Q_dev", Q_dev, n, ldq, m + 1)) return s;
    int mode = FOSI_REORTH_LOCAL_FULL;
    double tol = 1e-6;
    if (opts != nullptr) {
        if (opts->reorth_mode != 0) mode = opts->reorth_mode;
        if (opts->breakdown_tol > 0.0) tol = opts->breakdown_tol;
    }
    if (mode == FOSI_REORTH_SELECTIVE)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "the selective scheme is not available in the row-sharded run");
    if (mode != FOSI_REORTH_SINGLE && mode != FOSI_REORTH_TWICE && mode != FOSI_REORTH_LOCAL_FULL)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "unknown reorth_mode");
    const int passes = mode == FOSI_REORTH_SINGLE ? 1 : 2;
    *m_eff = 0;
    const Shards sh = make_shards(n, shards);
    int* flags = ctx->s.flags;
    if (fosi_status s = check_hip(ctx, hipMemsetAsync(flags, 0, 8 * sizeof(int), ctx->stream), "clear flags")) return s;

    // first column: every block scales its rows by the same 1 / ||v||
    sharded_dot(ctx, sh, nullptr, 0, 0, Q_dev, nullptr, nullptr, nullptr, ctx->s.coef_a, nullptr, 0, nullptr, nullptr, -1);
    launch_inv_sqrt(ctx, ctx->s.coef_a, ctx->s.scal + 1);
    for (int c = 0; c < sh.count; ++c) launch_scale(ctx, Q_dev + sh.begin[c], ctx->s.scal + 1, sh.rows(c), nullptr);

    for (int i = 0; i < m; ++i) {
        const float* q = Q_dev + (int64_t)i * ldq;
        float* h = Q_dev + (int64_t)(i + 1) * ldq;
        const int ncols = i + 1;
        if (mode == FOSI_REORTH_LOCAL_FULL) {
            const float* qprev = i > 0 ? q - ldq : nullptr;
            if (fosi_status s = sharded_operator(op, sh, q, h, qprev, true)) return s;
            sharded_dot(ctx, sh, Q_dev, ldq, ncols, h, q, qprev, ctx->s.scal + 4, ctx->s.coef_b, nullptr, 0, ctx->s.loc,
                        flags, FOSI_PROF_REORTH_DOT);
            if (ctx->tun.early_beta) {
                launch_lanczos_finalize_early(ctx, i, ctx->s.coef_b, ncols, tol);
                for (int c = 0; c < sh.count; ++c) {
                    const int64_t o = sh.begin[c], nr = sh.rows(c);
                    launch_combine_columns(ctx, Q_dev + o, ldq, ncols, ctx->s.coef_b, h + o, 1.0, nullptr, 0.0, nullptr, 0.0,
                                           nullptr, false, -1.0, h + o, nr, false, flags, FOSI_PROF_REORTH_SUB,
                                           (ncols + 2) * kVec * (double)nr, ctx->s.scal);
                }
                if (fosi_status s = launch_status(ctx, "sharded lanczos step")) return s;
                continue;
            }
            sharded_subtract(ctx, sh, Q_dev, ldq, ncols, ctx->s.coef_b, h, flags);
            launch_lanczos_finalize(ctx, i, sh.count, ctx->s.coef_b, ncols, nullptr, 0, ctx->s.loc + 2, tol, ctx->s.xchg3);
        } else {
            if (fosi_status s = sharded_operator(op, sh, q, h, nullptr, false)) return s;
            double* coef[2] = {ctx->s.coef_a, ctx->s.coef_b};
            for (int p = 0; p < passes; ++p) {
                sharded_dot(ctx, sh, Q_dev, ldq, ncols, h, nullptr, nullptr, nullptr, coef[p], nullptr, 0, nullptr, flags,
                            FOSI_PROF_REORTH_DOT);
                sharded_subtract(ctx, sh, Q_dev, ldq, ncols, coef[p], h, flags);
            }
            launch_lanczos_finalize(ctx, i, sh.count, ctx->s.coef_a, ncols, passes == 2 ? ctx->s.coef_b : nullptr,
                                    passes == 2 ? ncols : 0, nullptr, tol, ctx->s.xchg3);
        }
        for (int c = 0; c < sh.count; ++c) launch_scale(ctx, h + sh.begin[c], ctx->s.scal, sh.rows(c), flags);
        if (fosi_status s = launch_status(ctx, "sharded lanczos step")) return s;
    }

    int hflags[5] = {0, 0, 0, 0, 0};
    if (fosi_status s = check_hip(ctx, hipMemcpyAsync(alpha_host, ctx->s.alpha, sizeof(double) * m, hipMemcpyDeviceToHost,
                                                      ctx->stream), "copy alpha")) return s;
    if (fosi_status s = check_hip(ctx, hipMemcpyAsync(beta_host, ctx->s.beta, sizeof(double) * m, hipMemcpyDeviceToHost,
                                                      ctx->stream), "copy beta")) return s;
    if (fosi_status s = check_hip(ctx, hipMemcpyAsync(hflags, flags, sizeof(hflags), hipMemcpyDeviceToHost, ctx->stream),
                                  "copy flags")) return s;
    if (fosi_status s = check_hip(ctx, hipStreamSynchronize(ctx->stream), "lanczos synchronize")) return s;
    if (fosi_status s = check_hip(ctx, hipMemsetAsync(flags, 0, 8 * sizeof(int), ctx->stream), "clear flags")) return s;
    *m_eff = hflags[1];
    ctx->second_passes = hflags[4];
    if (hflags[0] == 2) return fail(ctx, FOSI_ERR_NONFINITE, "non-finite value in the Lanczos recurrence");
    return FOSI_OK;
}

/* ------------------------------------------------------------------- Eq. 8 */

fosi_status fosi_tridiag_eigh(int m, const double* alpha, const double* beta, double* evals, double* evecs) {
    if (m < 1 || alpha == nullptr || evals == nullptr || (m > 1 && beta == nullptr)) return FOSI_ERR_INVALID_ARG;
    for (int i = 0; i < m; ++i)
        if (!std::isfinite(alpha[i]) || (i + 1 < m && !std::isfinite(beta[i]))) return FOSI_ERR_NONFINITE;
    return tridiag_eigh(m, alpha, beta, evals, evecs) == 0 ? FOSI_OK : FOSI_ERR_NONFINITE;
}

static fosi_status fosi_ritz_impl(fosi_ctx* ctx, int64_t n, int m_eff, const float* Q_dev, int64_t ldq, const double* alpha_host,
                      const double* beta_host, int k, int l, float* V_dev, int64_t ldv, double* evals_host,
                      double* resid_host) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (alpha_host == nullptr || beta_host == nullptr || evals_host == nullptr)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "null argument");
    if (n < 1 || m_eff < 1 || k < 0 || l < 0) return fail(ctx, FOSI_ERR_INVALID_ARG, "bad sizes");
    if (m_eff > kMaxCols) return fail(ctx, FOSI_ERR_LIMIT, "m_eff exceeds FOSI_MAX_COLS");
    const int rv = k + l;
    if (rv < 1 || rv > m_eff) return fail(ctx, FOSI_ERR_RANK, "need 1 <= k + l <= m_eff");
    if (fosi_status s = check_matrix(ctx, "Q_dev", Q_dev, n, ldq, m_eff)) return s;
    if (fosi_status s = check_matrix(ctx, "V_dev", V_dev, n, ldv, rv)) return s;

    std::vector<double> u(m_eff), Z((size_t)m_eff * m_eff);
    if (fosi_status s = fosi_tridiag_eigh(m_eff, alpha_host, beta_host, u.data(), Z.data()))
        return fail(ctx, s, "tridiagonal eigen-solve failed");
    std::vector<int> sel(rv);
    for (int j = 0; j < k; ++j) sel[j] = m_eff - 1 - j;   // k largest, descending
    for (int j = 0; j < l; ++j) sel[k + j] = j;           // l smallest, ascending
    const double blast = std::fabs(beta_host[m_eff - 1]);
    for (int j = 0; j < rv; ++j) {
        evals_host[j] = u[sel[j]];
        if (resid_host != nullptr) resid_host[j] = blast * std::fabs(Z[(size_t)sel[j] * m_eff + (m_eff - 1)]);
    }
    // Ritz vectors on the matrix cores in 16-wide column blocks: up to 48 output columns per sweep of Q (64 when
    // that finishes the job in one sweep).  For comparison: the vector ALUs in chunks of at most 40 columns.
    const double vec = kVec * (double)n;
    const bool mfma = ctx->tun.ritz_mfma != 0;
    const int chunk = mfma ? (rv > 48 && rv <= 64 ? 64 : 48) : 40;
    for (int c0 = 0; c0 < rv; c0 += chunk) {
        const int cw = std::min(chunk, rv - c0);
        const int pad = mfma ? (cw + 15) / 16 * 16 : cw <= 8 ? 8 : cw <= 16 ? 16 : cw <= 24 ? 24 : cw <= 32 ? 32 : 40;
        // the coefficient block goes through the context's pinned staging buffer: the copy is asynchronous, and
        // the buffer is rewritten only after the previous copy out of it has finished
        if (fosi_status s = stage_acquire(ctx, ctx->stage_S_done, ctx->stage_S_busy)) return s;
        float* S = ctx->stage_S;
        for (int j = 0; j < m_eff; ++j)
            for (int t = 0; t < pad; ++t)
                S[(size_t)j * pad + t] = t < cw ? (float)Z[(size_t)sel[c0 + t] * m_eff + j] : 0.f;
        if (fosi_status s = check_hip(ctx, hipMemcpyAsync(ctx->s.S, S, sizeof(float) * (size_t)m_eff * pad,
                                                          hipMemcpyHostToDevice, ctx->stream), "upload S")) return s;
        if (fosi_status s = check_hip(ctx, hipEventRecord(ctx->stage_S_done, ctx->stream), "upload S")) return s;
        ctx->stage_S_busy = true;
        ProfScope ps(ctx, FOSI_PROF_RITZ_VECTORS, (m_eff + cw) * vec);
        if (mfma)
            launch_ritz_vectors_mfma(ctx, Q_dev, ldq, m_eff, ctx->s.S, cw, V_dev + (int64_t)c0 * ldv, ldv, n);
        else
            launch_ritz_vectors(ctx, Q_dev, ldq, m_eff, ctx->s.S, pad, cw, V_dev + (int64_t)c0 * ldv, ldv, n);
    }
    return launch_status(ctx, "ritz vectors");
}

/* ------------------------------------------------- Eq. 4 / Eq. 12 / Eq. 14 */

/* alpha / (a_j + sigma) (or with |a_j|) to device memory; unchanged between curvature refreshes, so it is
 * uploaded only when it differs from what the device already holds. */
static fosi_status upload_newton(fosi_ctx* ctx, int r_v, const double* evals_host, int curv_mode, double sigma,
                                 double alpha) {
    if (r_v <= 0) return FOSI_OK;
    double newton[kMaxCols];
    for (int j = 0; j < r_v; ++j) {
        const double a = curv_mode == FOSI_CURV_ABS ? std::fabs(evals_host[j]) : evals_host[j];
        const double den = a + sigma;
        if (!(std::fabs(den) >= 1e-30) || !std::isfinite(den))
            return fail(ctx, FOSI_ERR_NONFINITE, "Newton divisor a_j + sigma is zero or non-finite");
        newton[j] = alpha / den;
    }
    if (ctx->newton_cached != r_v || std::memcmp(newton, ctx->newton_cache, sizeof(double) * r_v) != 0) {
        // through the pinned staging buffer: no stream synchronisation, see fosi_ritz
        if (fosi_status s = stage_acquire(ctx, ctx->stage_newton_done, ctx->stage_newton_busy)) return s;
        std::memcpy(ctx->stage_newton, newton, sizeof(double) * r_v);
        if (fosi_status s = check_hip(ctx, hipMemcpyAsync(ctx->s.newton, ctx->stage_newton, sizeof(double) * r_v,
                                                          hipMemcpyHostToDevice, ctx->stream), "upload divisors"))
            return s;
        if (fosi_status s = check_hip(ctx, hipEventRecord(ctx->stage_newton_done, ctx->stream), "upload divisors")) return s;
        ctx->stage_newton_busy = true;
        std::memcpy(ctx->newton_cache, newton, sizeof(double) * r_v);
        ctx->newton_cached = r_v;
    }
    return FOSI_OK;
}

static fosi_status fosi_step_impl(fosi_ctx* ctx, int64_t n, int r_v, const float* V_dev, int64_t ldv, const double* evals_host,
                      const float* g_dev, const float* pi_dev, float* mom_dev, float* w_dev, const fosi_step_params* p) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (p == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, "params is null");
    if (n < 1 || r_v < 0) return fail(ctx, FOSI_ERR_INVALID_ARG, "bad sizes");
    if (r_v > kMaxCols) return fail(ctx, FOSI_ERR_LIMIT, "k + l exceeds FOSI_MAX_COLS");
    if (p->curv_mode != FOSI_CURV_SIGNED && p->curv_mode != FOSI_CURV_ABS)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "unknown curv_mode");
    if (fosi_status s = check_matrix(ctx, "V_dev", V_dev, n, ldv, r_v)) return s;
    if (r_v > 0 && evals_host == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, "evals_host is null");
    if (fosi_status s = check_vector(ctx, "g_dev", g_dev)) return s;
    if (fosi_status s = check_vector(ctx, "pi_dev", pi_dev, true)) return s;
    if (fosi_status s = check_vector(ctx, "mom_dev", mom_dev)) return s;
    if (fosi_status s = check_vector(ctx, "w_dev", w_dev)) return s;

    const double sigma = pi_dev != nullptr ? (double)p->sigma : 0.0;
    const double alpha = p->alpha, lr = p->lr, mu = p->momentum;
    if (fosi_status st = upload_newton(ctx, r_v, evals_host, p->curv_mode, sigma, alpha)) return st;
    const double vec = kVec * (double)n;
    const int extra = pi_dev != nullptr ? 1 : 0;
    // three sweeps of V: r_v + 1 (+1), r_v + 3 (+1), r_v + 3 vectors.  Timers: one bracket around the whole update, or
    // (when that class is not selected) one per sweep.
    const bool whole = ctx->prof_on && (ctx->prof_mask == 1 || ((ctx->prof_mask >> (FOSI_PROF_STEP + 1)) & 1) != 0);
    const int c1 = whole ? -1 : FOSI_PROF_STEP_PROJECT, c2 = whole ? -1 : FOSI_PROF_STEP_COMPLEMENT,
              c3 = whole ? -1 : FOSI_PROF_STEP_APPLY;
    if (whole) prof_begin(ctx, FOSI_PROF_STEP, r_v > 0 ? (3.0 * r_v + 7 + 2 * extra) * vec : (6.0 + extra) * vec);
    if (r_v > 0) {
        // c = V^T (g + pi)
        launch_dot_columns(ctx, V_dev, ldv, r_v, g_dev, pi_dev, nullptr, nullptr, n, ctx->s.coef_a, nullptr, 0, 1.0,
                           nullptr, nullptr, c1, (r_v + 1 + extra) * vec);
        // b <- momentum b + (g + pi) - V c ;  e = V^T b
        launch_complement_reproject(ctx, 0, V_dev, ldv, r_v, ctx->s.coef_a, g_dev, pi_dev, nullptr, mom_dev, nullptr,
                                    nullptr, n, mu, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, ctx->s.coef_b, c2,
                                    (r_v + 3 + extra) * vec);
        // d = newton . c - lr e
        launch_step_coefficients(ctx, r_v, lr);
    } else {
        // b <- momentum b + (g + pi)
        launch_combine_columns(ctx, V_dev, ldv, 0, ctx->s.coef_a, mom_dev, mu, g_dev, 1.0, pi_dev, 1.0, nullptr, false,
                               -1.0, mom_dev, n, false, nullptr, c2, (3.0 + extra) * vec);
    }
    // w <- w - lr b - V d   ( = w + Delta_1 + Delta_2 )
    launch_combine_columns(ctx, V_dev, ldv, r_v, ctx->s.coef_c, w_dev, 1.0, mom_dev, -lr, nullptr, 0.0, nullptr, false,
                           -1.0, w_dev, n, false, nullptr, c3, (r_v + 3) * vec);
    if (whole) prof_end(ctx);
    return launch_status(ctx, "fosi_step");
}

static fosi_status fosi_step_adamw_impl(fosi_ctx* ctx, int64_t n, int r_v, const float* V_dev, int64_t ldv,
                            const double* evals_host, const float* g_dev, const float* pi_dev, float* exp_avg_dev,
                            float* exp_avg_sq_dev, float* work_dev, float* w_dev, int64_t step_index,
                            const fosi_adamw_params* p) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (p == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, "params is null");
    if (n < 1 || r_v < 0 || step_index < 1) return fail(ctx, FOSI_ERR_INVALID_ARG, "bad sizes or step index");
    if (r_v > kMaxCols) return fail(ctx, FOSI_ERR_LIMIT, "k + l exceeds FOSI_MAX_COLS");
    if (p->curv_mode != FOSI_CURV_SIGNED && p->curv_mode != FOSI_CURV_ABS)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "unknown curv_mode");
    if (!(p->beta1 >= 0.f && p->beta1 < 1.f && p->beta2 >= 0.f && p->beta2 < 1.f))
        return fail(ctx, FOSI_ERR_INVALID_ARG, "beta1, beta2 must lie in [0, 1)");
    if (fosi_status s = check_matrix(ctx, "V_dev", V_dev, n, ldv, r_v)) return s;
    if (r_v > 0 && evals_host == nullptr) return fail(ctx, FOSI_ERR_INVALID_ARG, "evals_host is null");
    if (fosi_status s = check_vector(ctx, "g_dev", g_dev)) return s;
    if (fosi_status s = check_vector(ctx, "pi_dev", pi_dev, true)) return s;
    if (fosi_status s = check_vector(ctx, "exp_avg_dev", exp_avg_dev)) return s;
    if (fosi_status s = check_vector(ctx, "exp_avg_sq_dev", exp_avg_sq_dev)) return s;
    if (fosi_status s = check_vector(ctx, "work_dev", work_dev)) return s;
    if (fosi_status s = check_vector(ctx, "w_dev", w_dev)) return s;
    const double sigma = pi_dev != nullptr ? (double)p->sigma : 0.0;
    if (fosi_status st = upload_newton(ctx, r_v, evals_host, p->curv_mode, sigma, (double)p->alpha)) return st;
    const double b1 = p->beta1, b2 = p->beta2;
    const double inv_bc1 = 1.0 / (1.0 - std::pow(b1, (double)step_index));
    const double inv_bc2 = 1.0 / (1.0 - std::pow(b2, (double)step_index));
    const double vec = kVec * (double)n;
    const int extra = pi_dev != nullptr ? 1 : 0;
    // three sweeps of V: r_v + 1 (+1), r_v + 7 (+1), r_v + 3 vectors
    ProfScope ps(ctx, FOSI_PROF_STEP, r_v > 0 ? (3.0 * r_v + 11 + 2 * extra) * vec : (10.0 + extra) * vec);
    if (r_v > 0)   // c = V^T (g + pi)
        launch_dot_columns(ctx, V_dev, ldv, r_v, g_dev, pi_dev, nullptr, nullptr, n, ctx->s.coef_a, nullptr, 0, 1.0,
                           nullptr, nullptr, -1, 0.0);
    // moments of x = g + pi - V c, the optimiser's descent vector o, and e = V^T o
    launch_complement_reproject(ctx, 1, V_dev, ldv, r_v, ctx->s.coef_a, g_dev, pi_dev, w_dev, exp_avg_dev, exp_avg_sq_dev,
                                work_dev, n, 0.0, b1, b2, inv_bc1, inv_bc2, (double)p->eps, (double)p->lr,
                                (double)p->weight_decay, ctx->s.coef_b);
    if (r_v > 0) launch_step_coefficients_plus(ctx, r_v);   // d = newton . c + e
    // w <- w + o - V d   ( = w + Delta_1 + Delta_2 )
    launch_combine_columns(ctx, V_dev, ldv, r_v, ctx->s.coef_c, w_dev, 1.0, work_dev, 1.0, nullptr, 0.0, nullptr, false,
                           -1.0, w_dev, n, false, nullptr, -1, 0.0);
    return launch_status(ctx, "fosi_step_adamw");
}

/* ------------------------------------------------------ Algorithm 3 / Eq. 11 */

static fosi_status fosi_admm_begin_impl(fosi_ctx* ctx, int64_t n, float sigma, const float* pi_dev, float* w_anchor_dev,
                            float* wa_dev) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (n < 1 || !(sigma > 0.f)) return fail(ctx, FOSI_ERR_INVALID_ARG, "n and sigma must be positive");
    if (pi_dev == nullptr || w_anchor_dev == nullptr || wa_dev == nullptr)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "null argument");
    ProfScope ps(ctx, FOSI_PROF_ADMM, 4 * kVec * (double)n);
    launch_admm_begin(ctx, n, 1.0 / (double)sigma, pi_dev, w_anchor_dev, wa_dev);
    return launch_status(ctx, "admm_begin");
}

static fosi_status fosi_admm_end_impl(fosi_ctx* ctx, int64_t n, float sigma, const float* w_anchor_dev, const float* wa_dev,
                          float* pi_dev) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (n < 1 || !(sigma > 0.f)) return fail(ctx, FOSI_ERR_INVALID_ARG, "n and sigma must be positive");
    if (pi_dev == nullptr || w_anchor_dev == nullptr || wa_dev == nullptr)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "null argument");
    ProfScope ps(ctx, FOSI_PROF_ADMM, 4 * kVec * (double)n);
    launch_admm_end(ctx, n, (double)sigma, w_anchor_dev, wa_dev, pi_dev);
    return launch_status(ctx, "admm_end");
}

/* ------------------------------------------- measurement aid: memory-only sweep */

static fosi_status fosi_traffic_model_impl(fosi_ctx* ctx, int64_t n, const float* A_dev, int64_t lda, int cols_in,
                                           float* B_dev, int64_t ldb, int cols_out) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (n < 4 || (n & 3) != 0) return fail(ctx, FOSI_ERR_INVALID_ARG, "n must be a positive multiple of 4");
    if (cols_in < 0 || cols_out < 0 || cols_in + cols_out < 1) return fail(ctx, FOSI_ERR_INVALID_ARG, "bad column counts");
    if (fosi_status s = check_matrix(ctx, "A_dev", A_dev, n, lda, cols_in)) return s;
    if (fosi_status s = check_matrix(ctx, "B_dev", B_dev, n, ldb, cols_out)) return s;
    ProfScope ps(ctx, FOSI_PROF_TRAFFIC_MODEL, kVec * (double)n * (cols_in + cols_out));
    launch_traffic_model(ctx, A_dev, lda, cols_in, B_dev, ldb, cols_out, n, n > ((int64_t)8 << 20));
    return launch_status(ctx, "traffic model");
}

/* ------------------------------------------------------------------ timers */

static fosi_status fosi_profile_enable_impl(fosi_ctx* ctx, int on) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (on < 0) return fail(ctx, FOSI_ERR_INVALID_ARG, "bad profile selection");
    ctx->prof_on = on != 0;
    ctx->prof_mask = on;
    return FOSI_OK;
}

static fosi_status fosi_profile_reset_impl(fosi_ctx* ctx) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (fosi_status s = check_hip(ctx, hipStreamSynchronize(ctx->stream), "profile reset")) return s;
    for (auto& r : ctx->prof) {
        ctx->event_pool.push_back(r.start);
        ctx->event_pool.push_back(r.stop);
    }
    ctx->prof.clear();
    return FOSI_OK;
}

static fosi_status fosi_profile_read_impl(fosi_ctx* ctx, int kernel_class, int64_t* launches, double* total_ms,
                              double* algorithmic_bytes) {
    if (ctx == nullptr) return FOSI_ERR_INVALID_ARG;
    if (kernel_class < 0 || kernel_class >= FOSI_PROF_NUM || launches == nullptr || total_ms == nullptr ||
        algorithmic_bytes == nullptr)
        return fail(ctx, FOSI_ERR_INVALID_ARG, "bad profile query");
    if (fosi_status s = check_hip(ctx, hipStreamSynchronize(ctx->stream), "profile read")) return s;
    int64_t cnt = 0;
    double ms = 0.0, bytes = 0.0;
    for (auto& r : ctx->prof) {
        if (r.cls != kernel_class) continue;
        float t = 0.f;
        if (hipEventElapsedTime(&t, r.start, r.stop) != hipSuccess) continue;
        ++cnt;
        ms += t;
        bytes += r.bytes;
    }
    *launches = cnt;
    *total_ms = ms;
    *algorithmic_bytes = bytes;
    return FOSI_OK;
}


/* ---- the exported names: each runs its body behind the exception guard ---- */
fosi_status hvp_planted_create(fosi_ctx* ctx, int64_t n, int r, const float* U_dev, int64_t ldu,
                               const float* lam_dev, float shift, fosi_hvp** out) {
    return guarded(ctx, [&] { return hvp_planted_create_impl(ctx, n, r, U_dev, ldu, lam_dev, shift, out); });
}
fosi_status hvp_diag_create(fosi_ctx* ctx, int64_t n, const float* d_dev, fosi_hvp** out) {
    return guarded(ctx, [&] { return hvp_diag_create_impl(ctx, n, d_dev, out); });
}
fosi_status hvp_softmax_ggn_create(fosi_ctx* ctx, int B, int d, int C, const float* X_dev, const float* W_dev,
                                   fosi_hvp** out) {
    return guarded(ctx, [&] { return hvp_softmax_ggn_create_impl(ctx, B, d, C, X_dev, W_dev, out); });
}
fosi_status hvp_softmax_ggn_bf16_create(fosi_ctx* ctx, int B, int d, int C, const uint16_t* X_bf16_dev,
                                        const float* W_dev, fosi_hvp** out) {
    return guarded(ctx, [&] { return hvp_softmax_ggn_bf16_create_impl(ctx, B, d, C, X_bf16_dev, W_dev, out); });
}
fosi_status hvp_callback_create(fosi_ctx* ctx, int64_t n, fosi_hvp_fn fn, void* user, fosi_hvp** out) {
    return guarded(ctx, [&] { return hvp_callback_create_impl(ctx, n, fn, user, out); });
}
fosi_status hvp_apply(fosi_hvp* op, const float* v_dev, float* hv_dev) {
    return guarded(op != nullptr ? op->ctx : nullptr, [&] { return hvp_apply_impl(op, v_dev, hv_dev); });
}
fosi_status hvp_destroy(fosi_hvp* op) {
    return guarded(op != nullptr ? op->ctx : nullptr, [&] { return hvp_destroy_impl(op); });
}
fosi_status fosi_lanczos_begin(fosi_ctx* ctx, fosi_hvp* op, int64_t n, int m, float* Q_dev, int64_t ldq,
                               const fosi_lanczos_opts* opts) {
    return guarded(ctx, [&] { return fosi_lanczos_begin_impl(ctx, op, n, m, Q_dev, ldq, opts); });
}
fosi_status fosi_lanczos_end(fosi_ctx* ctx, double* alpha_host, double* beta_host, int32_t* m_eff) {
    return guarded(ctx, [&] { return fosi_lanczos_end_impl(ctx, alpha_host, beta_host, m_eff); });
}
fosi_status fosi_lanczos_row_sharded(fosi_ctx* ctx, fosi_hvp* op, int64_t n, int m, int shards, float* Q_dev,
                                     int64_t ldq, double* alpha_host, double* beta_host, int32_t* m_eff,
                                     const fosi_lanczos_opts* opts) {
    return guarded(ctx, [&] { return fosi_lanczos_row_sharded_impl(ctx, op, n, m, shards, Q_dev, ldq, alpha_host, beta_host, m_eff, opts); });
}
fosi_status fosi_ritz(fosi_ctx* ctx, int64_t n, int m_eff, const float* Q_dev, int64_t ldq, const double* alpha_host,
                      const double* beta_host, int k, int l, float* V_dev, int64_t ldv, double* evals_host,
                      double* resid_host) {
    return guarded(ctx, [&] { return fosi_ritz_impl(ctx, n, m_eff, Q_dev, ldq, alpha_host, beta_host, k, l, V_dev, ldv, evals_host, resid_host); });
}
fosi_status fosi_step(fosi_ctx* ctx, int64_t n, int r_v, const float* V_dev, int64_t ldv, const double* evals_host,
                      const float* g_dev, const float* pi_dev, float* mom_dev, float* w_dev, const fosi_step_params* p) {
    return guarded(ctx, [&] { return fosi_step_impl(ctx, n, r_v, V_dev, ldv, evals_host, g_dev, pi_dev, mom_dev, w_dev, p); });
}
fosi_status fosi_step_adamw(fosi_ctx* ctx, int64_t n, int r_v, const float* V_dev, int64_t ldv,
                            const double* evals_host, const float* g_dev, const float* pi_dev, float* exp_avg_dev,
                            float* exp_avg_sq_dev, float* work_dev, float* w_dev, int64_t step_index,
                            const fosi_adamw_params* p) {
    return guarded(ctx, [&] { return fosi_step_adamw_impl(ctx, n, r_v, V_dev, ldv, evals_host, g_dev, pi_dev, exp_avg_dev, exp_avg_sq_dev, work_dev, w_dev, step_index, p); });
}
fosi_status fosi_admm_begin(fosi_ctx* ctx, int64_t n, float sigma, const float* pi_dev, float* w_anchor_dev,
                            float* wa_dev) {
    return guarded(ctx, [&] { return fosi_admm_begin_impl(ctx, n, sigma, pi_dev, w_anchor_dev, wa_dev); });
}
fosi_status fosi_admm_end(fosi_ctx* ctx, int64_t n, float sigma, const float* w_anchor_dev, const float* wa_dev,
                          float* pi_dev) {
    return guarded(ctx, [&] { return fosi_admm_end_impl(ctx, n, sigma, w_anchor_dev, wa_dev, pi_dev); });
}
fosi_status fosi_traffic_model(fosi_ctx* ctx, int64_t n, const float* A_dev, int64_t lda, int cols_in, float* B_dev,
                               int64_t ldb, int cols_out) {
    return guarded(ctx, [&] { return fosi_traffic_model_impl(ctx, n, A_dev, lda, cols_in, B_dev, ldb, cols_out); });
}
fosi_status fosi_profile_enable(fosi_ctx* ctx, int on) {
    return guarded(ctx, [&] { return fosi_profile_enable_impl(ctx, on); });
}
fosi_status fosi_profile_reset(fosi_ctx* ctx) {
    return guarded(ctx, [&] { return fosi_profile_reset_impl(ctx); });
}
fosi_status fosi_profile_read(fosi_ctx* ctx, int kernel_class, int64_t* launches, double* total_ms,
                              double* algorithmic_bytes) {
    return guarded(ctx, [&] { return fosi_profile_read_impl(ctx, kernel_class, launches, total_ms, algorithmic_bytes); });
}

}  // extern "C"
