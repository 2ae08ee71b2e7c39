// fosi_step_noalloc: the model update of fosi_step for callers that cannot allocate device memory (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  It needs no context: the scratch
// memory the update's kernels use (partial sums, the coefficient vectors, the Newton factors) lives in a
// file-scope device array that every GPU holds from library load until the process ends.
#include <cmath>
#include <mutex>

#include "fosi_internal.h"

namespace {

using namespace fosi;

constexpr int kNoallocCols = FOSI_NOALLOC_MAX_COLS;
constexpr size_t kCols1 = kNoallocCols + 1;

// Layout of the array (byte offsets, every part 256-byte aligned).
constexpr size_t up256(size_t b) { return (b + 255) / 256 * 256; }
constexpr size_t kOffPartials = 0;                                                   // kMaxDotSlots x (cols + 1) doubles
constexpr size_t kOffCoefA = kOffPartials + up256(sizeof(double) * kMaxDotSlots * kCols1);
constexpr size_t kOffCoefB = kOffCoefA + up256(sizeof(double) * kCols1);
constexpr size_t kOffCoefC = kOffCoefB + up256(sizeof(double) * kCols1);
constexpr size_t kOffNewton = kOffCoefC + up256(sizeof(double) * kCols1);
constexpr size_t kOffScal = kOffNewton + up256(sizeof(double) * kCols1);              // 8 doubles
constexpr size_t kOffLoc = kOffScal + 256;                                           // 8 doubles
constexpr size_t kOffFlags = kOffLoc + 256;                                          // 8 ints
constexpr size_t kScratchBytes = kOffFlags + 256;
static_assert(kScratchBytes == FOSI_NOALLOC_SCRATCH_BYTES, "the header states the size of the array");

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// In host code `scratch` is only a stand-in for the symbol.  Its address on a GPU comes from hipGetSymbolAddress,
// asked once per device with that device current; each GPU has its own copy at its own address.
constexpr int kMaxDevices = 64;
std::mutex g_setup_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {nullptr};
int g_cu_count[kMaxDevices] = {0};

fosi_status scratch_for_current_device(unsigned char** ptr, int* cus) {
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return FOSI_ERR_HIP;
    if (device < 0 || device >= kMaxDevices) return FOSI_ERR_LIMIT;
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    if (g_scratch_ptr[device] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return FOSI_ERR_HIP;
        }
        int n_cu = 0;
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n_cu < 1) {
            (void)hipGetLastError();
            return FOSI_ERR_HIP;
        }
        g_cu_count[device] = n_cu;
        g_scratch_ptr[device] = static_cast<unsigned char*>(p);
    }
    *ptr = g_scratch_ptr[device];
    *cus = g_cu_count[device];
    return FOSI_OK;
}

// What must hold a defined value at the start of a call, written by a kernel (no memset, so that a caller may
// capture the call): the two unit scales of "g + pi", the arrival counter of the reduction's second stage, and the
// Newton factors alpha / (a_j + sigma), which travel as a kernel argument instead of a host-to-device copy.
struct NewtonFactors {
    double f[kNoallocCols];
};

__global__ void k_noalloc_prepare(double* __restrict__ newton, double* __restrict__ scal, int* __restrict__ flags,
                                  NewtonFactors nf, int rv) {
    const int t = threadIdx.x;
    if (t < rv) newton[t] = nf.f[t];
    if (t < 8) {
        scal[t] = (t == 2 || t == 3) ? 1.0 : 0.0;
        flags[t] = 0;
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" fosi_status fosi_step_noalloc(void* hip_stream, int64_t n, int r_v, const float* V_dev, int64_t ldv,
                                         const double* evals_host, const float* g_dev, const float* pi_dev,
                                         float* mom_dev, float* w_dev, const fosi_step_params* p) {
    if (p == nullptr || g_dev == nullptr || mom_dev == nullptr || w_dev == nullptr) return FOSI_ERR_INVALID_ARG;
    if (n < 1 || r_v < 0) return FOSI_ERR_INVALID_ARG;
    if (r_v > kNoallocCols) return FOSI_ERR_LIMIT;                 // more columns than the static array was sized for
    if (p->curv_mode != FOSI_CURV_SIGNED && p->curv_mode != FOSI_CURV_ABS) return FOSI_ERR_INVALID_ARG;
    if (r_v > 0 && (V_dev == nullptr || evals_host == nullptr)) return FOSI_ERR_INVALID_ARG;
    if (r_v > 0 && (ldv < n || (ldv & 3) != 0 || !aligned16(V_dev))) return FOSI_ERR_BAD_LAYOUT;
    if (!aligned16(g_dev) || !aligned16(mom_dev) || !aligned16(w_dev) || (pi_dev != nullptr && !aligned16(pi_dev)))
        return FOSI_ERR_BAD_LAYOUT;

    const double sigma = pi_dev != nullptr ? (double)p->sigma : 0.0;
    NewtonFactors nf{};
    for (int j = 0; j < r_v; ++j) {
        const double a = p->curv_mode == FOSI_CURV_ABS ? std::fabs(evals_host[j]) : evals_host[j];
        const double den = a + sigma;
        if (!(std::fabs(den) >= 1e-30) || !std::isfinite(den)) return FOSI_ERR_NONFINITE;
        nf.f[j] = (double)p->alpha / den;
    }

    unsigned char* base = nullptr;
    int cus = 0;
    if (fosi_status s = scratch_for_current_device(&base, &cus)) return s;

    // A context on the stack whose scratch pointers lead into the static array: the update's launchers take their
    // buffers from it exactly as they take them from an allocated context.  Launch shapes are the size-derived
    // defaults (no environment knobs here).
    fosi_ctx local;
    local.stream = static_cast<hipStream_t>(hip_stream);
    local.sm_count = cus;
    local.tun = Tunables{};
    local.tun.early_beta = 1;
    local.tun.ritz_mfma = 1;
    local.tun.step_waves_per_cu = 8;
    local.tun.step_cols_per_wave = 0;
    local.s = Scratch{};
    local.s.partials = reinterpret_cast<double*>(base + kOffPartials);
    local.s.norm_partials = local.s.partials;                      // not used by the update (no norm is requested)
    local.s.coef_a = reinterpret_cast<double*>(base + kOffCoefA);
    local.s.coef_b = reinterpret_cast<double*>(base + kOffCoefB);
    local.s.coef_c = reinterpret_cast<double*>(base + kOffCoefC);
    local.s.newton = reinterpret_cast<double*>(base + kOffNewton);
    local.s.scal = reinterpret_cast<double*>(base + kOffScal);
    local.s.loc = reinterpret_cast<double*>(base + kOffLoc);
    local.s.flags = reinterpret_cast<int*>(base + kOffFlags);
    fosi_ctx* ctx = &local;

    hipLaunchKernelGGL(k_noalloc_prepare, dim3(1), dim3(64), 0, ctx->stream, ctx->s.newton, ctx->s.scal, ctx->s.flags, nf,
                       r_v);
    const double lr = p->lr, mu = p->momentum;
    if (r_v > 0) {
        // c = V^T (g + pi);  b <- momentum b + (g + pi) - V c, e = V^T b;  d = newton . c - lr e
        launch_dot_columns(ctx, V_dev, ldv, r_v, g_dev, pi_dev, nullptr, nullptr, n, ctx->s.coef_a, nullptr, 0, 1.0,
                           nullptr, nullptr, -1, 0.0);
        launch_complement_reproject(ctx, 0, V_dev, ldv, r_v, ctx->s.coef_a, g_dev, pi_dev, nullptr, mom_dev, nullptr,
                                    nullptr, n, mu, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, ctx->s.coef_b);
        launch_step_coefficients(ctx, r_v, lr);
    } else {
        launch_combine_columns(ctx, V_dev, ldv, 0, ctx->s.coef_a, mom_dev, mu, g_dev, 1.0, pi_dev, 1.0, nullptr, false,
                               -1.0, mom_dev, n, false, nullptr, -1, 0.0);
    }
    // w <- w - lr b - V d   ( = w + Delta_1 + Delta_2 )
    launch_combine_columns(ctx, V_dev, ldv, r_v, ctx->s.coef_c, w_dev, 1.0, mom_dev, -lr, nullptr, 0.0, nullptr, false,
                           -1.0, w_dev, n, false, nullptr, -1, 0.0);
    return hipGetLastError() == hipSuccess ? FOSI_OK : FOSI_ERR_HIP;
}
