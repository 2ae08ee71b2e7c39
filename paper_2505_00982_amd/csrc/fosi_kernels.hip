// Streaming kernels of the curvature step and the update rule, written for
// gfx950 (64-lane wavefronts, 256 CUs in 8 XCDs, HBM-bound work).
//
// Two kernel families carry almost all of the traffic:
//   dot_columns      c = A^T x   for a tall column-major A (Gram-Schmidt
//                    coefficients of Algorithm 1, the planted operator's U^T v,
//                    the V^T g products of Eq. 4 / Eq. 12 / Eq. 14)
//   combine_columns  out = a0 y + a1 x1 + a2 x2 + sa A d   (h - Q c of Algorithm 1,
//                    the planted operator's U d + shift v, the V (.) terms of the
//                    update rule)
// Both stream every matrix element exactly once with 16-byte loads, multiply
// in fp64 (the product of two fp32 values is exact there) and round once when
// a vector is stored.  Cross-block sums are two-stage and in a fixed order, so
// results do not depend on scheduling.
#include <type_traits>

#include "fosi_internal.h"

namespace fosi {

namespace {

// 16-byte streaming load for matrix elements that are touched exactly once per sweep: marked
// non-temporal so that they do not displace the vectors (x, h, coefficients) that are re-read.
// On MI355X this alone lifts a pure read stream from ~6.2 to ~6.9 TB/s.
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream4(const float* p) {
    const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}

// Streaming store: on MI355X a plain store of the one output vector costs ~0.24 ms inside a 2 ms
// sweep of 13 GB (read/write turnarounds); marked non-temporal it costs ~0.1 ms.
__device__ __forceinline__ void store_stream4(float* p, const float4 v) {
    f32x4 t;
    t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
    __builtin_nontemporal_store(t, reinterpret_cast<f32x4*>(p));
}

// The same with device-scope write-through (sc1 + nt): the lines leave the L2 at once instead of lingering there
// as dirty streaming data.  Used where a kernel rewrites a vector in place and a long read-only sweep follows
// (the Gram-Schmidt subtraction before the operator's project sweep): with the plain streaming store that next
// sweep runs ~1.5 % slower while the L2s still write back (1.949 -> 1.921 ms on the 128-column project sweep of the
// n = 25.6 M workload; for the expand sweep's own output the two policies measure the same).  No builtin selects
// this combination of cache bits for a 16-byte store through a plain pointer, but the raw buffer store takes the
// bits as an operand: the store goes through a buffer descriptor (wave-uniform base and extent, per-lane byte
// offset) and stays an instruction the compiler schedules itself -- it, not this file, keeps the hardware's rule
// that the data registers of a store wider than 8 bytes are not overwritten within two wait states.  (An
// earlier version issued global_store_dwordx4 from an asm statement; the compiler could not see into it and
// scheduled such a write right behind it: corrupted elements at n = 25.6 M until padding was added by hand.)
// Stores beyond the descriptor's extent are dropped by the hardware.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kBufferStoreSc1Nt = 16 | 2;     // cache-policy operand of the raw buffer store: sc1 (bit 4), nt (bit 1)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t store_window(float* base, int64_t bytes) {
    // untyped 32-bit elements, no swizzle; the extent saturates below 4 GiB (callers pass at most one tile)
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, (int)(bytes < 0x7fffffff ? bytes : 0x7fffffff), 0x00020000);
}
__device__ __forceinline__ void store_through4(__amdgpu_buffer_rsrc_t window, uint32_t byte_offset, const float4 v) {
    f32x4 t;
    t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, t), window, (int)byte_offset, 0, kBufferStoreSc1Nt);
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// Sum over the 256 threads of a block; result valid in thread 0.
__device__ __forceinline__ double block_sum(double v, double* lds4) {
    v = wave_sum(v);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) lds4[wave] = v;
    __syncthreads();
    return lds4[0] + lds4[1] + lds4[2] + lds4[3];
}

// ---------------------------------------------------------------- dot_columns
// Work is split per wavefront: a wave owns a "slot" of up to JB (16 or 32) consecutive columns and sweeps
// float4 row groups (64 lanes x 4 rows) with a grid stride, keeping one fp64 accumulator per
// column.  Consecutive waves (of one XCD) own consecutive slots and walk the SAME rows, so the waves that
// share rows of the vector x sit in one workgroup or at least behind one L2, and no wave is idle
// whatever the number of slots.  The sweep is compiled for 4, 8, ..., JB columns; a slot whose width
// is not a multiple of 4 re-reads its last column for the (at most 3) padding positions, which hit
// in cache and are discarded.  partials[column * nrowlanes + rowlane] receives the wave's sums (the row
// lanes of a column are contiguous, so that the second stage reads them with coalesced loads), column
// index `ncols` the partial of sum(x^2) (from the waves of slot 0).

// One sweep of a slot compiled for NCOL columns (nc <= NCOL of them real).  `Aj0` points at row 0 of
// the slot's first column.  Everything but `lane` is uniform across the wave, so the column bases
// live in scalar registers and every load is "scalar base + one shared 32-bit lane offset".
template <int NCOL, int NX>
__device__ __forceinline__ void dot_sweep(const float* __restrict__ Aj0, int64_t lda, int nc,
                                          const float* __restrict__ x, const float* __restrict__ x2,
                                          const float* __restrict__ x3, double s2, double s3, int64_t t_begin,
                                          int64_t r_end, int64_t stride, int lane, bool do_xx, double* acc, double& xx) {
    // The vector's row group for the NEXT tile is requested while the current tile's columns are in
    // flight, so each trip of the loop costs one memory round trip, not two.
    float4 nx1 = make_float4(0.f, 0.f, 0.f, 0.f), nx2 = nx1, nx3 = nx1;
    uint32_t n_off = 0;
    bool n_ok = false;
    auto fetch_vector = [&](int64_t t) {
        // lanes past the end of a ragged last tile re-read its last row group and contribute zeros
        const int64_t rem = r_end - t;
        n_ok = lane < rem;
        n_off = (uint32_t)(n_ok ? lane : (int)rem - 1) << 4;      // bytes
        nx1 = *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(x + (t << 2)) + n_off);
        if (NX >= 2) nx2 = *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(x2 + (t << 2)) + n_off);
        if (NX >= 3) nx3 = *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(x3 + (t << 2)) + n_off);
    };
    if (t_begin < r_end) fetch_vector(t_begin);
    for (int64_t t = t_begin; t < r_end; t += stride) {
        const float4 xv = nx1, u2 = nx2, u3 = nx3;
        const uint32_t lane_bytes = n_off;
        const bool ok = n_ok;
        const float* At = Aj0 + (t << 2);
        float4 a[NCOL];
#pragma unroll
        for (int j = 0; j < NCOL; ++j) {
            const int col = j < nc ? j : nc - 1;
            a[j] = load_stream4(reinterpret_cast<const float*>(
                reinterpret_cast<const char*>(At + (int64_t)col * lda) + lane_bytes));
        }
        if (t + stride < r_end) fetch_vector(t + stride);
        double d0 = xv.x, d1 = xv.y, d2 = xv.z, d3 = xv.w;
        if (NX >= 2) {
            d0 = fma(s2, (double)u2.x, d0); d1 = fma(s2, (double)u2.y, d1);
            d2 = fma(s2, (double)u2.z, d2); d3 = fma(s2, (double)u2.w, d3);
        }
        if (NX >= 3) {
            d0 = fma(s3, (double)u3.x, d0); d1 = fma(s3, (double)u3.y, d1);
            d2 = fma(s3, (double)u3.z, d2); d3 = fma(s3, (double)u3.w, d3);
        }
        if (!ok) d0 = d1 = d2 = d3 = 0.0;
        if (do_xx) xx = fma(d0, d0, fma(d1, d1, fma(d2, d2, fma(d3, d3, xx))));
#pragma unroll
        for (int j = 0; j < NCOL; ++j)
            acc[j] = fma((double)a[j].x, d0, fma((double)a[j].y, d1, fma((double)a[j].z, d2, fma((double)a[j].w, d3, acc[j]))));
    }
}

// The vector is x (NX == 1), x + xs[0] x2 (NX == 2) or x + xs[0] x2 + xs[1] x3 (NX == 3), formed in fp64
// on the fly; xs points to device memory.
template <int JB, int NX>
__global__ __launch_bounds__(kThreads) void k_dot_columns(
    const float* __restrict__ A, int64_t lda, int ncols, const float* __restrict__ x,
    const float* __restrict__ x2, const float* __restrict__ x3, const double* __restrict__ xs, int64_t n,
    double* __restrict__ partials, int nslots, int nrowlanes, const int* __restrict__ stop) {
    static_assert(JB == 8 || JB == 16 || JB == 32, "the sweep variants below cover slots of up to 8, 16 or 32 columns");
    if (stop != nullptr && *stop != 0) return;
    const int lane = threadIdx.x & 63;
    // the wave index is the same for all 64 lanes: tell the compiler, so that the slot and its column
    // bases live in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // Waves are numbered within each XCD (the hardware deals workgroups to the 8 XCDs round-robin, and each
    // XCD has an L2 of its own): consecutive waves take consecutive column slots of the same row lane, so every
    // wave has work whatever the number of slots, and the waves that share rows of the vector x sit behind the
    // same L2 (x then comes from HBM once even when a row lane's slots span several workgroups).
    const int xcd = blockIdx.x & 7;
    const int lw = (int)(blockIdx.x >> 3) * 4 + wave;
    const int slot = lw % nslots;
    const int lane_in_xcd = lw / nslots;
    if (lane_in_xcd >= (nrowlanes >> 3)) return;        // spare waves of an XCD's last workgroup
    const int rowlane = lane_in_xcd * 8 + xcd;
    const int j0 = slot * JB;
    const int nc = max(0, min(JB, ncols - j0));
    const bool do_xx = (slot == 0);

    double acc[JB];
#pragma unroll
    for (int j = 0; j < JB; ++j) acc[j] = 0.0;
    double xx = 0.0;

    const int64_t n4 = n >> 2;
    // row groups are handed out round-robin over the row lanes; all uniform across the wave (float4 units)
    const int64_t t_begin = (int64_t)rowlane * 64;
    const int64_t r_end = n4;
    const int64_t stride = (int64_t)nrowlanes * 64;
    const double s2 = NX >= 2 ? xs[0] : 0.0, s3 = NX >= 3 ? xs[1] : 0.0;
    const float* Aj0 = A + (int64_t)j0 * lda;
#define FOSI_SWEEP(NC_) dot_sweep<NC_, NX>(Aj0, lda, nc, x, x2, x3, s2, s3, t_begin, r_end, stride, lane, do_xx, acc, xx)
    const int quads = (nc + 3) >> 2;
    if (quads == 0) {   // no columns (only reached by slot 0 when ncols == 0): just the sum of squares
        for (int64_t t = t_begin; t < r_end; t += stride) {
            if (t + lane < r_end) {
                const float4 xv = reinterpret_cast<const float4*>(x)[t + lane];
                double d0 = xv.x, d1 = xv.y, d2 = xv.z, d3 = xv.w;
                if (NX >= 2) {
                    const float4 u = reinterpret_cast<const float4*>(x2)[t + lane];
                    d0 = fma(s2, (double)u.x, d0); d1 = fma(s2, (double)u.y, d1);
                    d2 = fma(s2, (double)u.z, d2); d3 = fma(s2, (double)u.w, d3);
                }
                if (NX >= 3) {
                    const float4 u = reinterpret_cast<const float4*>(x3)[t + lane];
                    d0 = fma(s3, (double)u.x, d0); d1 = fma(s3, (double)u.y, d1);
                    d2 = fma(s3, (double)u.z, d2); d3 = fma(s3, (double)u.w, d3);
                }
                xx = fma(d0, d0, fma(d1, d1, fma(d2, d2, fma(d3, d3, xx))));
            }
        }
    } else if (quads == 1) {
        FOSI_SWEEP(4);
    } else if (quads == 2) {
        FOSI_SWEEP(8);
    } else if constexpr (JB >= 16) {       // a narrower kernel never gets here and keeps its smaller register count
        if (quads == 3) {
            FOSI_SWEEP(12);
        } else if (quads == 4) {
            FOSI_SWEEP(16);
        } else if constexpr (JB == 32) {
            if (quads == 5) FOSI_SWEEP(20);
            else if (quads == 6) FOSI_SWEEP(24);
            else if (quads == 7) FOSI_SWEEP(28);
            else FOSI_SWEEP(32);
        }
    }
#undef FOSI_SWEEP
    // the last (n mod 4) rows: one scalar row per lane of the first row group
    const int64_t tail_row = (n4 << 2) + lane;
    if (rowlane == 0 && lane < 3 && tail_row < n) {
        double dx = x[tail_row];
        if (NX >= 2) dx = fma(s2, (double)x2[tail_row], dx);
        if (NX >= 3) dx = fma(s3, (double)x3[tail_row], dx);
        if (do_xx) xx = fma(dx, dx, xx);
#pragma unroll
        for (int j = 0; j < JB; ++j)
            if (j < nc) acc[j] = fma((double)Aj0[(int64_t)j * lda + tail_row], dx, acc[j]);
    }

    double* pslot = partials + rowlane;
#pragma unroll
    for (int j = 0; j < JB; ++j) {
        if (j < nc) {                                   // uniform test: whole waves skip the padding columns
            const double v = wave_sum(acc[j]);
            if (lane == 0) pslot[(int64_t)(j0 + j) * nrowlanes] = v;
        }
    }
    if (do_xx) {
        const double v = wave_sum(xx);
        if (lane == 0) pslot[(int64_t)ncols * nrowlanes] = v;
    }
}

// End of one Lanczos step (Algorithm 1), shared by every kernel that finishes one: stores the diagonal entry a, the
// off-diagonal entry b and ||H q_step|| = hn, counts the step, raises the stop flag on a non-finite value (2) or
// on breakdown (1: b <= tol * hn) and leaves 1 / b for the normalisation.  Returns true when the run stops here.
__device__ __forceinline__ bool store_step_scalars(double a, double b, double hn, int step, double tol,
                                                   double* alpha, double* beta, double* hnorm, double* scal,
                                                   int* flags) {
    alpha[step] = a;
    beta[step] = b;
    hnorm[step] = hn;
    flags[1] = step + 1;
    const bool finite = (a - a == 0.0) && (b - b == 0.0) && (hn - hn == 0.0);
    const bool stops = !finite || !(b > tol * hn);
    if (!finite) flags[0] = 2;
    else if (stops) flags[0] = 1;
    scal[0] = 1.0 / b;
    return stops;
}

// sqrt of a difference of squares that rounding may have pushed below zero; NaN stays NaN
__device__ __forceinline__ double sqrt_clamped(double b2) { return b2 > 0.0 ? sqrt(b2) : (b2 == b2 ? 0.0 : b2); }

// What the last workgroup of the second stage does once every column sum is in memory (saves a launch).
struct ReduceTail {
    int kind;          // 0 none; 1 scalars of the local Gram-Schmidt pass; 2 end of a Lanczos step;
                       // 3 / 4: first / second pass of the 'selective' scheme
    int step;          // kinds 2-4: Lanczos step index
    double tol;        // kinds 2-4: breakdown tolerance
    double eta;        // kind 3: a second pass follows when the first one leaves less than eta * ||h||
    double* loc;       // kind 1: written {alpha~, beta~, ||h||^2}; kind 2: read
    double* neg;       // kind 1: written {-alpha~, -beta~}
    double* alpha;     // kind 2 outputs
    double* beta;
    double* hnorm;
    double* scal;      // kind 2: scal[0] = 1 / beta
    int* flags;        // [0] stop flag, [1] completed steps, [2] arrival counter of this kernel,
                       // [3] 'selective' scheme: non-zero = the second pass of this step is skipped,
                       // [4] 'selective' scheme: second passes done so far
};

// Second stage: one wavefront per output column sums the row-slot partials in a fixed order and applies
// the per-column scale.  Partial (slot, j) lives at partials[slot * slot_stride + j * col_stride].
// tail.kind != 0: every workgroup announces its result (release fence + counter); the one that arrives
// last reads all of `out` and finishes the step:
//   kind 1 (transposed product against [q_{i-1}, q_i] or [q_i], ncols = 2 or 1):
//          loc = {out[ncols-1], ncols > 1 ? out[0] : 0, out[ncols]}, neg = -loc[0..1];
//   kind 2 (end of a Lanczos step of the 'local_full' scheme): out holds the total coefficients (local +
//          full) of `ncols` columns and, in out[ncols], the squared norm of the vector x the full pass
//          worked on; loc = {alpha~, beta~, ||H q||^2} are the local parts of the last two coefficients.
//          x - Q c_full has squared norm ||x||^2 - ||c_full||^2 up to (Q^T Q - I) c_full . c_full, far below
//          fp64 rounding here, so beta is known BEFORE the subtraction sweep, which can then write the
//          normalised vector directly (no separate scaling sweep).
//   kind 3 (first pass of the 'selective' scheme, out = Q^T h and ||h||^2): the pass leaves
//          rho^2 = ||h||^2 - ||c||^2.  rho > eta ||h||: little was cancelled, the single pass is as good as it gets
//          in fp32 storage; the step ends here as in kind 2 and flags[3] = 1 makes the second pass's kernels
//          return at once.  Otherwise (the rounding error of the pass, ~eps ||h||, is large against what is
//          left) the subtraction writes h - Q c unscaled (scal[0] = 1), flags[3] = 0, and
//   kind 4 (second pass, out = Q^T h' and ||h'||^2) ends the step: alpha += c_i, beta from ||h'||^2 - ||c||^2.
__global__ __launch_bounds__(64) void k_reduce_columns(
    const double* __restrict__ partials, int nslots, int64_t slot_stride, int64_t col_stride, double* out,
    const float* __restrict__ scale, int nscale, double gscale, int ncols, const double* __restrict__ add_last2,
    const int* __restrict__ stop, ReduceTail tail) {
    if (stop != nullptr && *stop != 0) return;
    const int j = blockIdx.x, lane = threadIdx.x;
    const double* pj = partials + (int64_t)j * col_stride;
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    int slot = lane;
    for (; slot + 192 < nslots; slot += 256) {           // four independent loads in flight per lane
        const double v0 = pj[(int64_t)slot * slot_stride], v1 = pj[(int64_t)(slot + 64) * slot_stride];
        const double v2 = pj[(int64_t)(slot + 128) * slot_stride], v3 = pj[(int64_t)(slot + 192) * slot_stride];
        s0 += v0; s1 += v1; s2 += v2; s3 += v3;
    }
    for (; slot < nslots; slot += 64) s0 += pj[(int64_t)slot * slot_stride];
    double s = wave_sum((s0 + s1) + (s2 + s3));
    int last = 0;
    if (lane == 0) {
        if (j < ncols) {
            s *= gscale;
            if (scale != nullptr && j < nscale) s *= (double)scale[j];
            if (add_last2 != nullptr) {          // coefficients already removed along the last two columns
                if (j == ncols - 1) s += add_last2[0];
                if (j == ncols - 2) s += add_last2[1];
            }
        }
        out[j] = s;   // j == ncols: the plain sum of squares
        if (tail.kind != 0) {
            __threadfence();                                     // out[j] is visible before the arrival is
            last = atomicAdd(&tail.flags[2], 1) == (int)gridDim.x - 1;
        }
    }
    if (tail.kind == 0) return;
    last = __shfl(last, 0, 64);
    if (!last) return;
    __threadfence();                                             // the other workgroups' results are visible now
    if (lane == 0) tail.flags[2] = 0;                            // ready for the next launch
    if (tail.kind == 1) {
        if (lane == 0) {
            const double a = out[ncols - 1], b = ncols > 1 ? out[0] : 0.0;
            tail.loc[0] = a; tail.loc[1] = b; tail.loc[2] = out[ncols];
            tail.neg[0] = -a; tail.neg[1] = -b;
        }
        return;
    }
    if (tail.flags[0] != 0) return;
    const bool with_local = tail.kind == 2;
    double q = 0.0;
    for (int c = lane; c < ncols; c += 64) {
        double cf = out[c];
        if (with_local && c == ncols - 1) cf -= tail.loc[0];
        if (with_local && c == ncols - 2) cf -= tail.loc[1];
        q = fma(cf, cf, q);
    }
    q = wave_sum(q);
    if (lane == 0) {
        double a = out[ncols - 1];
        const double b = sqrt_clamped(out[ncols] - q);
        double hn;
        if (tail.kind == 2) hn = sqrt(tail.loc[2]);
        else if (tail.kind == 3) hn = sqrt(out[ncols]);
        else { hn = tail.hnorm[tail.step]; a += tail.alpha[tail.step]; }
        if (tail.kind == 3 && (b - b == 0.0) && (hn - hn == 0.0) && !(b > tail.eta * hn)) {
            // much was cancelled: the step ends in the second pass
            tail.alpha[tail.step] = a;
            tail.hnorm[tail.step] = hn;
            tail.scal[0] = 1.0;
            tail.flags[3] = 0;
            tail.flags[4] += 1;
            return;
        }
        const bool stops = store_step_scalars(a, b, hn, tail.step, tail.tol, tail.alpha, tail.beta, tail.hnorm,
                                              tail.scal, tail.flags);
        // 'selective': after a first pass that ends the step, or once the run has stopped, the second pass's
        // kernels (which test flags[3]) return at once; after a second pass its subtraction must still run
        if (tail.kind == 3 || (tail.kind == 4 && stops)) tail.flags[3] = 1;
    }
}

// s[q][0..3] = sum_j A[4 rows of row group rc[q], j] * d[j]  for the RPT row groups of one thread:
// columns in the outer loop, CU at a time, RPT*CU independent 16-byte streaming loads in flight.
template <int RPT, int CU>
__device__ __forceinline__ void accumulate_columns(const float* __restrict__ A, int64_t lda, int ncols,
                                                   const double* __restrict__ d, const int64_t* rc, double (*s)[4]) {
#pragma unroll
    for (int q = 0; q < RPT; ++q) s[q][0] = s[q][1] = s[q][2] = s[q][3] = 0.0;
    int j = 0;
    for (; j + CU <= ncols; j += CU) {
        float4 a[CU][RPT];
#pragma unroll
        for (int u = 0; u < CU; ++u)
#pragma unroll
            for (int q = 0; q < RPT; ++q) a[u][q] = load_stream4(A + (int64_t)(j + u) * lda + (rc[q] << 2));
#pragma unroll
        for (int u = 0; u < CU; ++u) {
            const double dj = d[j + u];
#pragma unroll
            for (int q = 0; q < RPT; ++q) {
                s[q][0] = fma((double)a[u][q].x, dj, s[q][0]);
                s[q][1] = fma((double)a[u][q].y, dj, s[q][1]);
                s[q][2] = fma((double)a[u][q].z, dj, s[q][2]);
                s[q][3] = fma((double)a[u][q].w, dj, s[q][3]);
            }
        }
    }
    for (; j < ncols; ++j) {
        const double dj = d[j];
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            const float4 av = load_stream4(A + (int64_t)j * lda + (rc[q] << 2));
            s[q][0] = fma((double)av.x, dj, s[q][0]);
            s[q][1] = fma((double)av.y, dj, s[q][1]);
            s[q][2] = fma((double)av.z, dj, s[q][2]);
            s[q][3] = fma((double)av.w, dj, s[q][3]);
        }
    }
}

// ------------------------------------------------------------ combine_columns
// out[row] = a0*y[row] + a1*x1[row] + a2*x2[row] + sa * sum_j A[row,j] d[j].
// A block owns RPT*1024 consecutive rows per iteration: every thread keeps RPT float4 row groups
// (256 rows apart) in fp64 accumulators and walks the columns in the outer loop, CU columns at a
// time, so RPT*CU independent 16-byte loads are in flight per thread and each column's page is
// touched in one burst (a workgroup that hops across all columns for every 4 KiB thrashes the
// address-translation caches).  d is read through uniform (scalar) loads.  With NORM the block's
// sum of out^2 (of the stored, rounded values) goes to norm_partials[blockIdx.x].
// oscale (device, may be null): factor applied to every element before the rounding, e.g. 1/beta.
// With LDOT (used by the planted operator inside a Lanczos run) the block also emits the partial sums
// of out.x1 and out.x3 (x3 may be null): norm_partials[{0,1,2} * gridDim.x + block] = {out^2, out.x1, out.x3}.
template <bool HAS_Y, bool HAS_X1, bool HAS_X2, bool NORM, bool LDOT, int RPT, int CU>
__global__ __launch_bounds__(kThreads) void k_combine_columns(
    const float* __restrict__ A, int64_t lda, int ncols, const double* __restrict__ d, const float* y,
    double a0, const float* __restrict__ x1, double a1, const float* __restrict__ x2, double a2,
    const float* __restrict__ x3, double sa, float* out, int64_t n, double* __restrict__ norm_partials,
    const double* __restrict__ oscale, const int* __restrict__ stop) {
    if (stop != nullptr && *stop != 0) return;
    __shared__ double red[4];
    const double osc = oscale != nullptr ? oscale[0] : 1.0;   // device-side factor applied to the whole result
    const int tid = threadIdx.x;
    const int64_t n4 = n >> 2;
    const int64_t tile = (int64_t)kThreads * RPT;
    const int64_t ntiles = (n4 + tile - 1) / tile;
    double nrm = 0.0, dot1 = 0.0, dot3 = 0.0;
    const int64_t t_begin = blockIdx.x, t_end = ntiles, t_step = gridDim.x;
    for (int64_t t = t_begin; t < t_end; t += t_step) {
        int64_t r4[RPT], rc[RPT];
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            r4[q] = t * tile + (int64_t)q * kThreads + tid;
            rc[q] = r4[q] < n4 ? r4[q] : n4 - 1;      // ragged last tile: re-read a valid row, discard below
        }
        // the vector operands of the epilogue are requested now, so that they travel while the columns stream
        float4 py[RPT], p1[RPT], p2[RPT], p3[RPT];
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            if (HAS_Y) py[q] = reinterpret_cast<const float4*>(y)[rc[q]];
            if (HAS_X1) p1[q] = reinterpret_cast<const float4*>(x1)[rc[q]];
            if (HAS_X2) p2[q] = reinterpret_cast<const float4*>(x2)[rc[q]];
            if (LDOT && x3 != nullptr) p3[q] = reinterpret_cast<const float4*>(x3)[rc[q]];
        }
        double s[RPT][4];
        accumulate_columns<RPT, CU>(A, lda, ncols, d, rc, s);
        // this tile's part of the output as a store window (uniform: t is the same in every lane)
        const int64_t tile_groups = n4 - t * tile < tile ? n4 - t * tile : tile;
        const __amdgpu_buffer_rsrc_t window = store_window(out + ((t * tile) << 2), tile_groups << 4);
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            if (r4[q] >= n4) continue;
            double o0 = sa * s[q][0], o1 = sa * s[q][1], o2 = sa * s[q][2], o3 = sa * s[q][3];
            if (HAS_Y) {
                const float4 v = py[q];
                o0 = fma(a0, (double)v.x, o0); o1 = fma(a0, (double)v.y, o1);
                o2 = fma(a0, (double)v.z, o2); o3 = fma(a0, (double)v.w, o3);
            }
            float4 v1 = make_float4(0.f, 0.f, 0.f, 0.f);
            if (HAS_X1) {
                v1 = p1[q];
                o0 = fma(a1, (double)v1.x, o0); o1 = fma(a1, (double)v1.y, o1);
                o2 = fma(a1, (double)v1.z, o2); o3 = fma(a1, (double)v1.w, o3);
            }
            if (HAS_X2) {
                const float4 v = p2[q];
                o0 = fma(a2, (double)v.x, o0); o1 = fma(a2, (double)v.y, o1);
                o2 = fma(a2, (double)v.z, o2); o3 = fma(a2, (double)v.w, o3);
            }
            if (oscale != nullptr) { o0 *= osc; o1 *= osc; o2 *= osc; o3 *= osc; }
            const float4 o = make_float4((float)o0, (float)o1, (float)o2, (float)o3);
            if (HAS_Y) store_through4(window, (uint32_t)((q * kThreads + tid) << 4), o);   // in-place rewrite, a read sweep follows
            else store_stream4(out + (r4[q] << 2), o);
            if (NORM || LDOT) nrm = fma((double)o.x, (double)o.x, fma((double)o.y, (double)o.y,
                                    fma((double)o.z, (double)o.z, fma((double)o.w, (double)o.w, nrm))));
            if (LDOT) {
                dot1 = fma((double)o.x, (double)v1.x, fma((double)o.y, (double)v1.y,
                       fma((double)o.z, (double)v1.z, fma((double)o.w, (double)v1.w, dot1))));
                if (x3 != nullptr) {
                    const float4 v3 = p3[q];
                    dot3 = fma((double)o.x, (double)v3.x, fma((double)o.y, (double)v3.y,
                           fma((double)o.z, (double)v3.z, fma((double)o.w, (double)v3.w, dot3))));
                }
            }
        }
    }
    const int64_t tail_row = (n4 << 2) + tid;
    if (blockIdx.x == 0 && tid < 3 && tail_row < n) {
        double s = 0.0;
        for (int j = 0; j < ncols; ++j) s = fma((double)A[(int64_t)j * lda + tail_row], d[j], s);
        double o = sa * s;
        if (HAS_Y) o = fma(a0, (double)y[tail_row], o);
        if (HAS_X1) o = fma(a1, (double)x1[tail_row], o);
        if (HAS_X2) o = fma(a2, (double)x2[tail_row], o);
        if (oscale != nullptr) o *= osc;
        const float of = (float)o;
        out[tail_row] = of;
        if (NORM || LDOT) nrm = fma((double)of, (double)of, nrm);
        if (LDOT) {
            dot1 = fma((double)of, (double)x1[tail_row], dot1);
            if (x3 != nullptr) dot3 = fma((double)of, (double)x3[tail_row], dot3);
        }
    }
    if (LDOT) {
        const double b0 = block_sum(nrm, red), b1 = block_sum(dot1, red), b3 = block_sum(dot3, red);
        if (tid == 0) {
            norm_partials[blockIdx.x] = b0;
            norm_partials[(int64_t)gridDim.x + blockIdx.x] = b1;
            norm_partials[2 * (int64_t)gridDim.x + blockIdx.x] = b3;
        }
    } else if (NORM) {
        const double b = block_sum(nrm, red);
        if (tid == 0) norm_partials[blockIdx.x] = b;
    }
}

// ------------------------------------------------- complement + base optimiser + re-projection
// Second sweep of the update (Eq. 12 / Eq. 14), fused with the transposed product that the last sweep
// needs, so that V is streamed three times per update and not four:
//   x = g (+ pi) - V c                         (c = V^T (g + pi) from the first sweep)
//   heavy ball (OPT == 0):  b <- mu b + x ;                               z = b
//   AdamW      (OPT == 1):  m <- b1 m + (1-b1) x ;  v <- b2 v + (1-b2) x^2 ;
//                           o = -lr ( (m / bc1) / (sqrt(v / bc2) + eps) + wd w ) ;   z = o
//   e_j = sum_rows V[row, j] z[row]            (z as stored, i.e. rounded to fp32)
// A row of z needs every column of that row, and e_j needs that z again.  The S waves of a block
// therefore share one tile of 64 float4 row groups and split the columns: wave s keeps its (at most
// MAXC) columns of the tile in registers, the partial sums of V c are exchanged through LDS (added in a
// fixed order, so all waves hold identical values), every wave evaluates the optimiser for the tile and
// wave 0 stores its state, then each wave accumulates the e_j of its own columns from the registers.
// partials[j * gridDim.x + block] receives the block's part of e_j.
struct OptScalars {
    double mu;                                   // heavy ball
    double b1, b2, inv_bc1, inv_bc2, eps, lr, wd;   // AdamW (bc1, bc2: bias corrections of this step)
};

// The optimiser state of a row is read by every wave of the block and overwritten by wave 0: the reads
// must have returned before the block's barrier.  An empty volatile statement that consumes the loaded
// value cannot move across the barrier and forces the wait in front of it.
__device__ __forceinline__ void consume_before_barrier(float v) { asm volatile("" : : "v"(v)); }

template <int OPT>
__device__ __forceinline__ float optimiser_row(const OptScalars& p, double x, double w_, float& m_, float& v_) {
    if (OPT == 0) {
        m_ = (float)fma(p.mu, (double)m_, x);
        return m_;
    }
    const double mn = p.b1 * (double)m_ + (1.0 - p.b1) * x;
    const double vn = p.b2 * (double)v_ + (1.0 - p.b2) * x * x;
    m_ = (float)mn;
    v_ = (float)vn;
    return (float)(-p.lr * ((mn * p.inv_bc1) / (sqrt(vn * p.inv_bc2) + p.eps) + p.wd * w_));
}

// All waves of a block run the same width NCOL >= cw (columns per wave); positions past a wave's last
// real column re-read that column (cache hits) and are discarded.  pi may be null.
template <int OPT, int NCOL>
__global__ __launch_bounds__(512) void k_complement_reproject(
    const float* __restrict__ V, int64_t ldv, int ncols, int cw, const double* __restrict__ c,
    const float* __restrict__ g, const float* __restrict__ pi, const float* __restrict__ w, float* m, float* v,
    float* __restrict__ o_out, int64_t n, OptScalars p, double* __restrict__ partials) {
    extern __shared__ double exch[];             // [2][S][4][64]: partial sums of V c, double buffered
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int S = (int)(blockDim.x >> 6);
    const int j0 = wave * cw;                    // this wave's columns: [j0, j0 + nc), nc >= 1 unless ncols == 0
    const int nc = max(0, min(cw, ncols - j0));
    const float* Vj0 = V + (int64_t)j0 * ldv;
    const int64_t n4 = n >> 2;
    const int64_t ntiles = (n4 + 63) >> 6;
    const bool has_pi = pi != nullptr;

    double acc[NCOL];
    double cj[NCOL];                             // this wave's coefficients (uniform), zero for the padding
#pragma unroll
    for (int j = 0; j < NCOL; ++j) {
        acc[j] = 0.0;
        cj[j] = j < nc ? c[j0 + j] : 0.0;
    }
    int par = 0;

    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        // everything but `lane` is uniform: tile base in scalar registers, one 32-bit lane offset for all loads
        const int64_t base = t << 8;             // first row of the tile
        const int64_t rem = n4 - (t << 6);       // row groups left (> 0)
        const bool ok = lane < rem;              // ragged last tile: other lanes re-read its last group, add zeros
        const uint32_t lane_bytes = (uint32_t)(ok ? lane : (int)(rem < 64 ? rem : 64) - 1) << 4;
        auto vec4 = [&](const float* x) {
            return *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(x + base) + lane_bytes);
        };
        const float4 pg = vec4(g);
        // no branch around a load: without pi the gradient is read again (a cache hit) and dropped, so that all
        // loads of the tile are issued back to back
        float4 pp = vec4(has_pi ? pi : g), pw = make_float4(0.f, 0.f, 0.f, 0.f), pv = pw;
        if (!has_pi) pp = pw;
        float4 pm = vec4(m);
        if (OPT == 1) {
            pw = vec4(w);
            pv = vec4(v);
        }
        float4 a[NCOL];
        const float* Vt = Vj0 + base;
        if (nc > 0) {                            // uniform; with no columns at all (ncols == 0) V may be null
#pragma unroll
            for (int j = 0; j < NCOL; ++j) {
                const int col = j < nc ? j : nc - 1;
                a[j] = load_stream4(reinterpret_cast<const float*>(
                    reinterpret_cast<const char*>(Vt + (int64_t)col * ldv) + lane_bytes));
            }
        } else {
#pragma unroll
            for (int j = 0; j < NCOL; ++j) a[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
        for (int j = 0; j < NCOL; ++j) {
            s0 = fma((double)a[j].x, cj[j], s0); s1 = fma((double)a[j].y, cj[j], s1);
            s2 = fma((double)a[j].z, cj[j], s2); s3 = fma((double)a[j].w, cj[j], s3);
        }
        // keep the tile as fp32 across the exchange: without this the compiler holds the fp64 conversions of
        // all columns (twice the registers) for the second use below
#pragma unroll
        for (int j = 0; j < NCOL; ++j)
            asm volatile("" : "+v"(a[j].x), "+v"(a[j].y), "+v"(a[j].z), "+v"(a[j].w));
        if (S > 1) {
            double* mine = exch + (((par * S + wave) << 2) << 6) + lane;
            mine[0] = s0; mine[64] = s1; mine[128] = s2; mine[192] = s3;
            consume_before_barrier(pm.x);
            if (OPT == 1) consume_before_barrier(pv.x);
            __syncthreads();
            s0 = s1 = s2 = s3 = 0.0;
            for (int q = 0; q < S; ++q) {
                const double* o = exch + (((par * S + q) << 2) << 6) + lane;
                s0 += o[0]; s1 += o[64]; s2 += o[128]; s3 += o[192];
            }
            par ^= 1;                            // the next tile writes the other half: one barrier per tile suffices
        }
        double x0 = (double)pg.x - s0, x1 = (double)pg.y - s1, x2 = (double)pg.z - s2, x3 = (double)pg.w - s3;
        if (has_pi) { x0 += (double)pp.x; x1 += (double)pp.y; x2 += (double)pp.z; x3 += (double)pp.w; }
        float4 z;
        z.x = optimiser_row<OPT>(p, x0, (double)pw.x, pm.x, pv.x);
        z.y = optimiser_row<OPT>(p, x1, (double)pw.y, pm.y, pv.y);
        z.z = optimiser_row<OPT>(p, x2, (double)pw.z, pm.z, pv.z);
        z.w = optimiser_row<OPT>(p, x3, (double)pw.w, pm.w, pv.w);
        if (wave == 0 && ok) {
            float* mo = reinterpret_cast<float*>(reinterpret_cast<char*>(m + base) + lane_bytes);
            if (OPT == 0) {
                store_stream4(mo, pm);
            } else {
                *reinterpret_cast<float4*>(mo) = pm;
                *reinterpret_cast<float4*>(reinterpret_cast<char*>(v + base) + lane_bytes) = pv;
                store_stream4(reinterpret_cast<float*>(reinterpret_cast<char*>(o_out + base) + lane_bytes), z);
            }
        }
        const double z0 = ok ? (double)z.x : 0.0, z1 = ok ? (double)z.y : 0.0;
        const double z2 = ok ? (double)z.z : 0.0, z3 = ok ? (double)z.w : 0.0;
#pragma unroll
        for (int j = 0; j < NCOL; ++j)
            acc[j] = fma((double)a[j].x, z0, fma((double)a[j].y, z1, fma((double)a[j].z, z2,
                     fma((double)a[j].w, z3, acc[j]))));
    }

    // the last (n mod 4) rows: block 0, one row per lane; every wave evaluates them, wave 0 stores
    if (blockIdx.x == 0) {
        const int64_t tail_row = (n4 << 2) + lane;
        const bool tl = lane < 3 && tail_row < n;
        float mm = 0.f, vv = 0.f, zz = 0.f;
        if (tl) {
            double sacc = 0.0;
            for (int j = 0; j < ncols; ++j) sacc = fma((double)V[(int64_t)j * ldv + tail_row], c[j], sacc);
            double x = (double)g[tail_row] - sacc;
            if (has_pi) x += (double)pi[tail_row];
            mm = m[tail_row];
            if (OPT == 1) vv = v[tail_row];
            zz = optimiser_row<OPT>(p, x, OPT == 1 ? (double)w[tail_row] : 0.0, mm, vv);
        }
        if (S > 1) {
            consume_before_barrier(zz);
            __syncthreads();
        }
        if (tl) {
            if (wave == 0) {
                m[tail_row] = mm;
                if (OPT == 1) { v[tail_row] = vv; o_out[tail_row] = zz; }
            }
#pragma unroll
            for (int j = 0; j < NCOL; ++j)
                if (j < nc) acc[j] = fma((double)Vj0[(int64_t)j * ldv + tail_row], (double)zz, acc[j]);
        }
    }

    double* pblock = partials + blockIdx.x;
#pragma unroll
    for (int j = 0; j < NCOL; ++j) {
        if (j < nc) {                            // uniform test
            const double e = wave_sum(acc[j]);
            if (lane == 0) pblock[(int64_t)(j0 + j) * gridDim.x] = e;
        }
    }
    if (wave == 0 && lane == 0) pblock[(int64_t)ncols * gridDim.x] = 0.0;   // the reduction kernel also sums this (unused) slot
}

// d_j = newton_j c_j + e_j  (AdamW variant of the last sweep's coefficients: w += o - V d)
__global__ void k_step_coefficients_plus(const double* __restrict__ c, const double* __restrict__ e,
                                         const double* __restrict__ newton, int rv, double* __restrict__ dcoef) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < rv) dcoef[j] = newton[j] * c[j] + e[j];
}

// ---------------------------------------------------------------- small kernels
// End of one Lanczos step (Algorithm 1): diagonal entry, off-diagonal entry,
// breakdown / non-finite detection, reciprocal for the normalisation.
__global__ __launch_bounds__(kThreads) void k_lanczos_finalize(
    const double* __restrict__ norm_partials, int norm_slots, const double* __restrict__ coef_a,
    const double* __restrict__ coef_b, int cols_a, int cols_b, const double* __restrict__ hh_ptr, int step,
    double tol, double* __restrict__ alpha,
    double* __restrict__ beta, double* __restrict__ hnorm, double* __restrict__ scal, int* flags) {
    if (flags[0] != 0) return;
    __shared__ double red[4];
    double s = 0.0;
    for (int i = threadIdx.x; i < norm_slots; i += kThreads) s += norm_partials[i];
    s = block_sum(s, red);
    if (threadIdx.x == 0) {
        double a = coef_a[cols_a - 1];             // coefficient along the current vector, first pass
        if (cols_b > 0) a += coef_b[cols_b - 1];   // ... and second pass
        const double b = sqrt(s);
        // ||H q_step||^2 before orthogonalisation: by-product of the first pass, or handed in
        const double hn = sqrt(hh_ptr != nullptr ? hh_ptr[0] : coef_a[cols_a]);
        store_step_scalars(a, b, hn, step, tol, alpha, beta, hnorm, scal, flags);
    }
}

// End of a Lanczos step when the full pass only removes rounding-level components (the local pass has
// taken the rest): c holds the total coefficients (local + full) for `cols` columns and, in c[cols], the
// squared norm of the vector x the full pass worked on; loc = {alpha~, beta~, ||H q||^2} are the local
// parts added to the last two coefficients.  Then x - Q c_full has squared norm ||x||^2 - ||c_full||^2
// up to (Q^T Q - I) c_full . c_full, far below fp64 rounding here, so beta is known BEFORE the
// subtraction sweep, which can then write the normalised vector directly (no separate scaling sweep).
__global__ __launch_bounds__(kThreads) void k_lanczos_finalize_early(
    const double* __restrict__ c, int cols, const double* __restrict__ loc, int step, double tol,
    double* __restrict__ alpha, double* __restrict__ beta, double* __restrict__ hnorm, double* __restrict__ scal,
    int* flags) {
    if (flags[0] != 0) return;
    __shared__ double red[4];
    double s = 0.0;
    for (int j = threadIdx.x; j < cols; j += kThreads) {
        double cf = c[j];
        if (j == cols - 1) cf -= loc[0];
        if (j == cols - 2) cf -= loc[1];
        s = fma(cf, cf, s);
    }
    s = block_sum(s, red);
    if (threadIdx.x == 0) {
        store_step_scalars(c[cols - 1], sqrt_clamped(c[cols] - s), sqrt(loc[2]), step, tol, alpha, beta, hnorm, scal,
                           flags);
    }
}

// Fixed-order sum over `nslots` partial sums of one quantity (element i at p[i * stride]) by the 256 threads of
// a block: four independent loads per thread and trip, then the block sum.  Result valid in thread 0.
__device__ __forceinline__ double block_sum_strided(const double* __restrict__ p, int nslots, int64_t stride, double* red) {
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    int i = threadIdx.x;
    for (; i + 3 * kThreads < nslots; i += 4 * kThreads) {
        const double v0 = p[(int64_t)i * stride], v1 = p[(int64_t)(i + kThreads) * stride];
        const double v2 = p[(int64_t)(i + 2 * kThreads) * stride], v3 = p[(int64_t)(i + 3 * kThreads) * stride];
        s0 += v0; s1 += v1; s2 += v2; s3 += v3;
    }
    for (; i < nslots; i += kThreads) s0 += p[(int64_t)i * stride];
    return block_sum((s0 + s1) + (s2 + s3), red);
}

// Sums the {out^2, out.x1, out.x3} partials of the operator's expand sweep: loc = {alpha~, beta~, ||h||^2},
// neg = {-alpha~, -beta~} (the scales with which q_i and q_{i-1} enter the vector of the full pass).
// Partial w of slot i lives at parts[w * wstride + i * sstride].  One workgroup of 1024 threads: the partials
// were written by other compute units, every load is a trip to memory, so all loads of a thread (a few slots
// x 3) are issued before the first sum.
constexpr int kLocalThreads = 1024;
__global__ __launch_bounds__(kLocalThreads) void k_reduce_local(const double* __restrict__ parts, int nslots,
                                                                 int64_t wstride, int64_t sstride,
                                                                 double* __restrict__ loc, double* __restrict__ neg,
                                                                 const int* __restrict__ stop) {
    if (stop != nullptr && *stop != 0) return;
    __shared__ double red[3][kLocalThreads / 64];
    double s0 = 0.0, s1 = 0.0, s3 = 0.0;
    int i = threadIdx.x;
    for (; i + 3 * kLocalThreads < nslots; i += 4 * kLocalThreads) {       // 12 independent loads per trip
        double v[4][3];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int w = 0; w < 3; ++w) v[u][w] = parts[w * wstride + (int64_t)(i + u * kLocalThreads) * sstride];
#pragma unroll
        for (int u = 0; u < 4; ++u) { s0 += v[u][0]; s1 += v[u][1]; s3 += v[u][2]; }
    }
    for (; i < nslots; i += kLocalThreads) {
        const double v0 = parts[(int64_t)i * sstride], v1 = parts[wstride + (int64_t)i * sstride];
        const double v2 = parts[2 * wstride + (int64_t)i * sstride];
        s0 += v0; s1 += v1; s3 += v2;
    }
    s0 = wave_sum(s0); s1 = wave_sum(s1); s3 = wave_sum(s3);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { red[0][wave] = s0; red[1][wave] = s1; red[2][wave] = s3; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t0 = 0.0, t1 = 0.0, t3 = 0.0;
        for (int q = 0; q < kLocalThreads / 64; ++q) { t0 += red[0][q]; t1 += red[1][q]; t3 += red[2][q]; }
        loc[0] = t1; loc[1] = t3; loc[2] = t0;
        neg[0] = -t1; neg[1] = -t3;
    }
}

// dst[w] = sum over slots of parts[w * nslots + slot], w < width <= 3 (fixed order).
__global__ __launch_bounds__(kThreads) void k_fold_partials(const double* __restrict__ parts, int nslots, int width,
                                                            double* __restrict__ dst, const int* __restrict__ stop) {
    if (stop != nullptr && *stop != 0) return;
    __shared__ double red[4];
    for (int w = 0; w < width; ++w) {
        const double s = block_sum_strided(parts + (int64_t)w * nslots, nslots, 1, red);
        if (threadIdx.x == 0) dst[w] = s;
    }
}

// Same outputs from a transposed product against [q_{i-1}, q_i] (nc == 2) or [q_i] (nc == 1).
__global__ void k_local_from_coef(const double* __restrict__ coef, int nc, double* __restrict__ loc,
                                  double* __restrict__ neg, const int* __restrict__ stop) {
    if (stop != nullptr && *stop != 0) return;
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        const double a = coef[nc - 1], b = nc > 1 ? coef[0] : 0.0;
        loc[0] = a; loc[1] = b; loc[2] = coef[nc];
        neg[0] = -a; neg[1] = -b;
    }
}

__global__ void k_inv_sqrt(const double* in, double* out) {
    if (threadIdx.x == 0 && blockIdx.x == 0) out[0] = 1.0 / sqrt(in[0]);
}

__global__ __launch_bounds__(kThreads) void k_scale(float* x, const double* __restrict__ factor, int64_t n,
                                                    const int* __restrict__ stop) {
    if (stop != nullptr && *stop != 0) return;
    const double f = factor[0];
    const int64_t n4 = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t r4 = (int64_t)blockIdx.x * kThreads + threadIdx.x; r4 < n4; r4 += stride) {
        float4 v = reinterpret_cast<float4*>(x)[r4];
        v.x = (float)((double)v.x * f); v.y = (float)((double)v.y * f);
        v.z = (float)((double)v.z * f); v.w = (float)((double)v.w * f);
        reinterpret_cast<float4*>(x)[r4] = v;
    }
    const int64_t tail_row = (n4 << 2) + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x < 3 && tail_row < n) x[tail_row] = (float)((double)x[tail_row] * f);
}

__global__ __launch_bounds__(kThreads) void k_diag_apply(const float* __restrict__ d, const float* __restrict__ v,
                                                         float* __restrict__ out, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) out[i] = d[i] * v[i];
}

// Ritz vectors (Eq. 8): V[:, t] = sum_j Q[:, j] S[j, t].  S is m x RV row-major
// (zero padded to RV columns) and read through uniform loads; every thread keeps
// 4 rows x RV outputs in registers and streams Q once.
template <int RV>
__global__ __launch_bounds__(kThreads) void k_ritz_vectors(
    const float* __restrict__ Q, int64_t ldq, int m, const float* __restrict__ S, int rv,
    float* __restrict__ V, int64_t ldv, int64_t n) {
    const int64_t n4 = n >> 2;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t r4 = (int64_t)blockIdx.x * kThreads + threadIdx.x; r4 < n4; r4 += stride) {
        float4 acc[RV];
#pragma unroll
        for (int t = 0; t < RV; ++t) acc[t] = make_float4(0.f, 0.f, 0.f, 0.f);
        int j = 0;
        for (; j + 2 <= m; j += 2) {
            const float4 q0 = load_stream4(Q + (int64_t)j * ldq + (r4 << 2));
            const float4 q1 = load_stream4(Q + (int64_t)(j + 1) * ldq + (r4 << 2));
            const float* s0 = S + (int64_t)j * RV;
            const float* s1 = s0 + RV;
#pragma unroll
            for (int t = 0; t < RV; ++t) {
                const float c0 = s0[t], c1 = s1[t];
                acc[t].x = fmaf(q1.x, c1, fmaf(q0.x, c0, acc[t].x));
                acc[t].y = fmaf(q1.y, c1, fmaf(q0.y, c0, acc[t].y));
                acc[t].z = fmaf(q1.z, c1, fmaf(q0.z, c0, acc[t].z));
                acc[t].w = fmaf(q1.w, c1, fmaf(q0.w, c0, acc[t].w));
            }
        }
        for (; j < m; ++j) {
            const float4 q0 = load_stream4(Q + (int64_t)j * ldq + (r4 << 2));
            const float* s0 = S + (int64_t)j * RV;
#pragma unroll
            for (int t = 0; t < RV; ++t) {
                const float c0 = s0[t];
                acc[t].x = fmaf(q0.x, c0, acc[t].x);
                acc[t].y = fmaf(q0.y, c0, acc[t].y);
                acc[t].z = fmaf(q0.z, c0, acc[t].z);
                acc[t].w = fmaf(q0.w, c0, acc[t].w);
            }
        }
#pragma unroll
        for (int t = 0; t < RV; ++t)
            if (t < rv) reinterpret_cast<float4*>(V + (int64_t)t * ldv)[r4] = acc[t];
    }
    const int64_t tail_row = (n4 << 2) + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x < 3 && tail_row < n) {
        for (int t = 0; t < rv; ++t) {
            float s = 0.f;
            for (int j = 0; j < m; ++j) s = fmaf(Q[(int64_t)j * ldq + tail_row], S[(int64_t)j * RV + t], s);
            V[(int64_t)t * ldv + tail_row] = s;
        }
    }
}

// The same product on the matrix cores, for up to CB * 16 output columns (CB = 1..4).  It is a dense contraction
// at 11-14 flop per byte, above what the vector ALUs sustain at HBM speed without packed fp32 (the kernel above
// reaches ~60 % of the HBM rate), but within reach of v_mfma_f32_16x16x4_f32: 16-wide column blocks pad 30 columns
// to 32 and 40 to 48 (2 n m 48 flop at n = 125 M, m = 100 is 7.6 ms of matrix work against a memory floor of
// 8.8 ms; 32-wide tiles would pad 40 to 64 and be bound by the matrix cores).  The product is taken transposed, so
// that a lane ends up with float4 stores of consecutive rows and no transpose is needed.
// Per instruction: V^T tile (16 output columns x 16 rows) += S^T (16 x 4) . Q^T (4 x 16 rows).
// Lane l = 16 g + i feeds S[k0 + g][16 cb + i] (from LDS) and, as the other operand, one of the four rows of its
// 16-byte load of Lanczos column k0 + g (rows 4 i + c, c = 0..3 of a 64-row group: four instructions share one
// load; a load instruction covers 4 columns x 256 contiguous bytes); accumulator register v of the instruction
// for row c is output column 16 cb + 4 g + v, so the four instructions of one (cb, row group) give float4 stores of
// 4 consecutive rows per output column.  A wave owns RG row groups of 64 rows; U k-steps (of 4 columns) per
// register set, two sets, so that 2 U RG loads per lane are in flight while the matrix instructions run.
// S: m x (16 CB) row-major, zero padded.  LDS rows are pitched so that the four 16-lane groups of a read hit
// distinct banks.
typedef float floatx4 __attribute__((ext_vector_type(4)));

template <int CB>
constexpr int ritz16_pitch() { return CB <= 3 ? 48 : 80; }      // = 16 mod 64 banks

template <int CB, int RG, int U>
__global__ __launch_bounds__(kThreads) void k_ritz_vectors_mfma16(
    const float* __restrict__ Q, int64_t ldq, int m, const float* __restrict__ S, int rv,
    float* __restrict__ V, int64_t ldv, int64_t n) {
    constexpr int SP = ritz16_pitch<CB>();
    extern __shared__ float Ssh[];                 // (m rounded up to 4) x SP, rows beyond m and padding columns zero
    const int tid = threadIdx.x;
    const int mp = (m + 3) & ~3;
    for (int i = tid; i < mp * SP; i += kThreads) {
        const int row = i / SP, col = i - row * SP;
        Ssh[i] = (row < m && col < CB * 16) ? S[row * (CB * 16) + col] : 0.f;
    }
    __syncthreads();
    const int lane = tid & 63, i16 = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane((int)(tid >> 6));
    const int64_t n4 = n >> 2;
    const int64_t ntiles = (n4 + RG * 16 - 1) / (RG * 16);
    for (int64_t tile = (int64_t)blockIdx.x * 4 + wave; tile < ntiles; tile += (int64_t)gridDim.x * 4) {
        int64_t rgi[RG];
        bool ok[RG];
        const float* qp[RG];
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            rgi[r] = (tile * RG + r) * 16 + i16;   // this lane's float4 row group in sub-tile r
            ok[r] = rgi[r] < n4;
            qp[r] = Q + ((ok[r] ? rgi[r] : n4 - 1) << 2);
        }
        floatx4 acc[CB][RG][4];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int r = 0; r < RG; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[cb][r][c] = floatx4{0.f, 0.f, 0.f, 0.f};
        auto issue = [&](int kb, float4 (*q)[RG]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (kb + 4 * u < mp) {             // uniform
                    const int k = min(kb + 4 * u + g, m - 1);   // padding columns re-read the last one, times 0
#pragma unroll
                    for (int r = 0; r < RG; ++r) q[u][r] = load_stream4(qp[r] + (int64_t)k * ldq);
                }
            }
        };
        auto multiply = [&](int kb, const float4 (*q)[RG]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (kb + 4 * u < mp) {
                    float a[CB];
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) a[cb] = Ssh[(kb + 4 * u + g) * SP + cb * 16 + i16];
#pragma unroll
                    for (int r = 0; r < RG; ++r)
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb) {
                            acc[cb][r][0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[cb], q[u][r].x, acc[cb][r][0], 0, 0, 0);
                            acc[cb][r][1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[cb], q[u][r].y, acc[cb][r][1], 0, 0, 0);
                            acc[cb][r][2] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[cb], q[u][r].z, acc[cb][r][2], 0, 0, 0);
                            acc[cb][r][3] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[cb], q[u][r].w, acc[cb][r][3], 0, 0, 0);
                        }
                }
            }
        };
        float4 qa[U][RG], qb[U][RG];
        issue(0, qa);
        for (int k0 = 0; k0 < mp; k0 += 8 * U) {
            issue(k0 + 4 * U, qb);
            __builtin_amdgcn_sched_barrier(0);
            multiply(k0, qa);
            __builtin_amdgcn_sched_barrier(0);
            issue(k0 + 8 * U, qa);
            __builtin_amdgcn_sched_barrier(0);
            multiply(k0 + 4 * U, qb);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            if (!ok[r]) continue;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int col = cb * 16 + 4 * g + v;
                    if (col < rv)
                        store_stream4(V + (int64_t)col * ldv + (rgi[r] << 2),
                                      make_float4(acc[cb][r][0][v], acc[cb][r][1][v], acc[cb][r][2][v], acc[cb][r][3][v]));
                }
        }
    }
    const int64_t tail_row = (n4 << 2) + tid;
    if (blockIdx.x == 0 && tid < 3 && tail_row < n) {
        for (int t = 0; t < rv; ++t) {
            float s = 0.f;
            for (int j = 0; j < m; ++j) s = fmaf(Q[(int64_t)j * ldq + tail_row], Ssh[j * SP + t], s);
            V[(int64_t)t * ldv + tail_row] = s;
        }
    }
}

// Coefficients of the last sweep of the update (Eq. 4 / Eq. 12 / Eq. 14):
//   d_j = newton_j * c_j  -  lr * e_j ,  c = V^T (g + pi),  e = V^T b,
// so that  w += -lr b - V d  equals  w + Delta_1 + Delta_2.
__global__ void k_step_coefficients(const double* __restrict__ c, const double* __restrict__ e,
                                    const double* __restrict__ newton, double lr, int rv,
                                    double* __restrict__ dcoef) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < rv) dcoef[j] = newton[j] * c[j] - lr * e[j];
}

// Algorithm 3: anchor = w_a + pi / sigma; w_a = anchor.
__global__ __launch_bounds__(kThreads) void k_admm_begin(int64_t n, double inv_sigma, const float* __restrict__ pi,
                                                         float* __restrict__ anchor, float* wa) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        const float v = (float)fma((double)pi[i], inv_sigma, (double)wa[i]);
        anchor[i] = v;
        wa[i] = v;
    }
}

// Algorithm 3 / Eq. 11: pi += sigma (w_a - anchor).
__global__ __launch_bounds__(kThreads) void k_admm_end(int64_t n, double sigma, const float* __restrict__ anchor,
                                                       const float* __restrict__ wa, float* pi) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride)
        pi[i] = (float)fma(sigma, (double)wa[i] - (double)anchor[i], (double)pi[i]);
}


int elementwise_grid(int64_t work_items) {
    int64_t g = (work_items + kThreads - 1) / kThreads;
    if (g < 1) g = 1;
    if (g > kMaxNormSlots) g = kMaxNormSlots;
    return (int)g;
}

ReduceTail make_tail(fosi_ctx* ctx, int kind, int step, double tol) {
    ReduceTail t{};
    t.kind = kind;
    t.step = step;
    t.tol = tol;
    t.eta = ctx->reorth_eta;
    t.loc = ctx->s.loc;
    t.neg = ctx->s.scal + 4;
    t.alpha = ctx->s.alpha;
    t.beta = ctx->s.beta;
    t.hnorm = ctx->s.hnorm;
    t.scal = ctx->s.scal;
    t.flags = ctx->s.flags;
    return t;
}

void dot_columns_launch(fosi_ctx* ctx, const float* A, int64_t lda, int ncols, const float* x, const float* x2,
                        const float* x3, const double* xs, int64_t n, double* coef, const float* scale, int nscale,
                        double gscale, const double* add_last2, const int* stop, int prof_cls, double prof_bytes,
                        int tail_kind, int tail_step, double tail_tol) {
    const int64_t n4 = n >> 2;
    // Columns per wave: 32 (216-230 registers, two waves per SIMD), 16 (120-134, three to four) or 8.  Measured on
    // MI355X: 16 is never slower than 32 (n = 25.6 M: 430.3 against 431.9 ms per step of workload 4; n = 2^20:
    // 10.1 against 11.2 ms of workload 2); 8 wins below a few million rows, where a wave makes only a handful of
    // trips (9.8 ms at n = 2^20) and loses a little on the large workloads' Gram-Schmidt products.
    int JB = ctx->tun.dot_slot_cols;
    if (JB != 8 && JB != 16 && JB != 32) JB = n <= ((int64_t)1 << 22) ? 8 : 16;
    const int nslots = ncols > 0 ? (ncols + JB - 1) / JB : 1;
    // row lanes (a multiple of 8, one share per XCD): as many as the targeted number of resident waves allows, not
    // more than the row groups of 256 rows (rounded up to 8; a row lane without rows contributes zeros)
    // Waves in flight: two workgroups (8 waves) per CU up to 8 M rows; beyond, one (4 waves, each with 16+ loads of
    // 1 KiB in flight, sweeping twice as many rows) is faster: n = 25.6 M project sweep 1.916 -> 1.908 ms,
    // Gram-Schmidt product 0.626 -> 0.618 ms; at n = 1 M it costs 2.5 %.  Counts that are not a power of two times
    // the slot count leave row lanes uneven (320 workgroups: +22 %).
    const int target_blocks = ctx->tun.dot_target_blocks > 0 ? ctx->tun.dot_target_blocks
                              : (n >= ((int64_t)1 << 23) ? ctx->sm_count : 2 * ctx->sm_count);
    int64_t per_xcd = ((int64_t)target_blocks * 4 / 8) / nslots;
    const int64_t groups = (n4 + 63) / 64;
    if (per_xcd > (groups + 7) / 8) per_xcd = (groups + 7) / 8;
    if (per_xcd > kMaxDotSlots / 8) per_xcd = kMaxDotSlots / 8;
    if (per_xcd < 1) per_xcd = 1;
    const int rowslots = (int)per_xcd * 8;
    const int64_t blocks_per_xcd = (per_xcd * nslots + 3) / 4;
    dim3 grid((unsigned)(blocks_per_xcd * 8));
    if (prof_cls >= 0) prof_begin(ctx, prof_cls, prof_bytes);
    if (x2 != nullptr && xs == nullptr) xs = ctx->s.scal + 2;   // plain sum of the vectors: scales 1, 1
#define FOSI_DOT(JB_, NX_)                                                                                          \
    hipLaunchKernelGGL((k_dot_columns<JB_, NX_>), grid, dim3(kThreads), 0, ctx->stream, A, lda, ncols, x, x2, x3, xs, n, \
                       ctx->s.partials, nslots, rowslots, stop)
    if (JB == 8) {
        if (x3 != nullptr) FOSI_DOT(8, 3);
        else if (x2 != nullptr) FOSI_DOT(8, 2);
        else FOSI_DOT(8, 1);
    } else if (JB == 16) {
        if (x3 != nullptr) FOSI_DOT(16, 3);
        else if (x2 != nullptr) FOSI_DOT(16, 2);
        else FOSI_DOT(16, 1);
    } else {
        if (x3 != nullptr) FOSI_DOT(32, 3);
        else if (x2 != nullptr) FOSI_DOT(32, 2);
        else FOSI_DOT(32, 1);
    }
#undef FOSI_DOT
    if (prof_cls >= 0) prof_end(ctx);
    hipLaunchKernelGGL(k_reduce_columns, dim3(ncols + 1), dim3(64), 0, ctx->stream, ctx->s.partials, rowslots, (int64_t)1,
                       (int64_t)rowslots, coef, scale, nscale, gscale, ncols, add_last2, stop,
                       make_tail(ctx, tail_kind, tail_step, tail_tol));
}

}  // namespace

void launch_dot_columns(fosi_ctx* ctx, const float* A, int64_t lda, int ncols, const float* x, const float* x2,
                        const float* x3, const double* xs, int64_t n, double* coef, const float* scale, int nscale,
                        double gscale, const double* add_last2, const int* stop, int prof_cls, double prof_bytes,
                        int tail_kind, int tail_step, double tail_tol) {
    dot_columns_launch(ctx, A, lda, ncols, x, x2, x3, xs, n, coef, scale, nscale, gscale, add_last2, stop, prof_cls,
                       prof_bytes, tail_kind, tail_step, tail_tol);
}

namespace {

template <int RPT, int CU>
int combine_columns_cfg(fosi_ctx* ctx, const float* A, int64_t lda, int ncols, const double* d, const float* y,
                        double a0, const float* x1, double a1, const float* x2, double a2, const float* x3,
                        bool local_dots, double sa, float* out, int64_t n, bool want_norm, const int* stop,
                        int prof_cls, double prof_bytes, const double* oscale) {
    const int64_t n4 = n >> 2;
    const int64_t tile = (int64_t)kThreads * RPT;
    int64_t g = (n4 + tile - 1) / tile;
    if (g < 1) g = 1;
    if (g > kMaxNormSlots) g = kMaxNormSlots;
    if (ctx->tun.comb_max_blocks > 0 && g > ctx->tun.comb_max_blocks) g = ctx->tun.comb_max_blocks;
    const int grid = (int)g;
    if (prof_cls >= 0) prof_begin(ctx, prof_cls, prof_bytes);
#define FOSI_COMBINE(Y, X1, X2, NRM, LD)                                                                         \
    hipLaunchKernelGGL((k_combine_columns<Y, X1, X2, NRM, LD, RPT, CU>), dim3(grid), dim3(kThreads), 0, ctx->stream, \
                       A, lda, ncols, d, y, a0, x1, a1, x2, a2, x3, sa, out, n, ctx->s.norm_partials, oscale, stop)
    const bool hy = y != nullptr, h1 = x1 != nullptr, h2 = x2 != nullptr;
    if (!hy && h1 && !h2 && !want_norm && local_dots) FOSI_COMBINE(false, true, false, false, true);   // expand + local dots
    else if (!hy && h1 && !h2 && !want_norm) FOSI_COMBINE(false, true, false, false, false);     // operator expand
    else if (hy && !h1 && !h2 && want_norm) FOSI_COMBINE(true, false, false, true, false);       // Gram-Schmidt subtract
    else if (hy && h1 && !h2 && !want_norm) FOSI_COMBINE(true, true, false, false, false);       // momentum / apply
    else if (hy && h1 && h2 && !want_norm) FOSI_COMBINE(true, true, true, false, false);         // momentum with dual
    else if (hy && !h1 && !h2 && !want_norm) FOSI_COMBINE(true, false, false, false, false);
    else FOSI_COMBINE(true, true, true, true, false);  // not reached by the library; kept total
#undef FOSI_COMBINE
    if (prof_cls >= 0) prof_end(ctx);
    return grid;
}

}  // namespace

int launch_combine_columns(fosi_ctx* ctx, const float* A, int64_t lda, int ncols, const double* d, const float* y,
                           double a0, const float* x1, double a1, const float* x2, double a2, const float* x3,
                           bool local_dots, double sa, float* out, int64_t n, bool want_norm, const int* stop,
                           int prof_cls, double prof_bytes, const double* oscale) {
#define FOSI_CFG(R, C)                                                                                            \
    return combine_columns_cfg<R, C>(ctx, A, lda, ncols, d, y, a0, x1, a1, x2, a2, x3, local_dots, sa, out, n,     \
                                     want_norm, stop, prof_cls, prof_bytes, oscale)
    switch (ctx->tun.comb_rows_per_thread * 100 + ctx->tun.comb_cols_unroll) {
        case 108: FOSI_CFG(1, 8);
        case 116: FOSI_CFG(1, 16);
        case 204: FOSI_CFG(2, 4);
        case 208: FOSI_CFG(2, 8);
        case 402: FOSI_CFG(4, 2);
        case 404: FOSI_CFG(4, 4);
        case 408: FOSI_CFG(4, 8);
        case 802: FOSI_CFG(8, 2);
        case 803: FOSI_CFG(8, 3);
        case 804: FOSI_CFG(8, 4);
        default: break;
    }
    // Not set (or not one of the shapes above): two shapes.  Small: 4 row groups x 8 columns in flight per thread,
    // tiles of 4096 rows, three workgroups per CU.  Large: 8 x 4, tiles of 8192 rows (32 KiB per column visit), one
    // workgroup per CU (250-370 registers).  The large shape streams 1.5-3 % faster per byte (MI355X, whole steps:
    // n = 25.6 M 427.5 -> 422.2 ms, n = 125 M 2756 -> 2695 ms together with the product's wave count; n = 2-12 M
    // 0.5-3 %), but with one workgroup per CU its tiles come in rounds of one per CU: at n = 1 M half the CUs would
    // get no tile (6 % slower), and a count just above a whole number of rounds wastes most of a round.  So: large
    // when there are many rounds (the hardware's dispatch evens them out), or when its rounds cost no more than the
    // small shape's half-size tiles spread over the CUs (2 % dearer per byte).
    // Other shapes measured at n = 25.6 M: 8 x 1 ... 8 x 3, 6 x 2, 6 x 4, 12 x 2, 16 x 1 within 0.6 % of 8 x 4 or slower.
    {
        const int64_t cus = ctx->sm_count > 0 ? ctx->sm_count : 1;
        const int64_t large_tiles = (n + 8191) / 8192;
        const int64_t large_rounds = (large_tiles + cus - 1) / cus;              // in large-tile times
        const int64_t small_halves = (2 * large_tiles + cus - 1) / cus;          // half-size tiles on the busiest CU
        if (large_rounds >= 8 || 100 * large_rounds <= 51 * small_halves) FOSI_CFG(8, 4);
    }
    FOSI_CFG(4, 8);
#undef FOSI_CFG
}

void launch_lanczos_finalize(fosi_ctx* ctx, int step, int norm_slots, const double* coef_a, int cols_a,
                             const double* coef_b, int cols_b, const double* hh, double tol, const double* norm_parts) {
    hipLaunchKernelGGL(k_lanczos_finalize, dim3(1), dim3(kThreads), 0, ctx->stream,
                       norm_parts != nullptr ? norm_parts : ctx->s.norm_partials, norm_slots,
                       coef_a, coef_b, cols_a, cols_b, hh, step, tol, ctx->s.alpha, ctx->s.beta, ctx->s.hnorm,
                       ctx->s.scal, ctx->s.flags);
}

void launch_lanczos_finalize_early(fosi_ctx* ctx, int step, const double* coef, int cols, double tol) {
    hipLaunchKernelGGL(k_lanczos_finalize_early, dim3(1), dim3(kThreads), 0, ctx->stream, coef, cols, ctx->s.loc, step, tol,
                       ctx->s.alpha, ctx->s.beta, ctx->s.hnorm, ctx->s.scal, ctx->s.flags);
}

void launch_reduce_local(fosi_ctx* ctx, int nslots, const int* stop, const double* parts) {
    // the expand sweep leaves [3][nslots]; a caller's buffer holds one {out^2, out.x1, out.x3} triple per slot
    if (parts == nullptr)
        hipLaunchKernelGGL(k_reduce_local, dim3(1), dim3(kLocalThreads), 0, ctx->stream, ctx->s.norm_partials, nslots,
                           (int64_t)nslots, (int64_t)1, ctx->s.loc, ctx->s.scal + 4, stop);
    else
        hipLaunchKernelGGL(k_reduce_local, dim3(1), dim3(kLocalThreads), 0, ctx->stream, parts, nslots, (int64_t)1,
                           (int64_t)3, ctx->s.loc, ctx->s.scal + 4, stop);
}

void launch_fold_partials(fosi_ctx* ctx, int nslots, int width, double* dst, const int* stop) {
    hipLaunchKernelGGL(k_fold_partials, dim3(1), dim3(kThreads), 0, ctx->stream, ctx->s.norm_partials, nslots, width,
                       dst, stop);
}

void launch_reduce_shards(fosi_ctx* ctx, int shards, int ncols, double* coef, const float* scale, int nscale,
                          double gscale, const double* add_last2, const int* stop) {
    hipLaunchKernelGGL(k_reduce_columns, dim3(ncols + 1), dim3(64), 0, ctx->stream, ctx->s.xchg, shards,
                       (int64_t)(kMaxCols + 1), (int64_t)1, coef, scale, nscale, gscale, ncols, add_last2, stop,
                       make_tail(ctx, 0, 0, 0.0));
}

void launch_local_from_coef(fosi_ctx* ctx, const double* coef, int nc, const int* stop) {
    hipLaunchKernelGGL(k_local_from_coef, dim3(1), dim3(64), 0, ctx->stream, coef, nc, ctx->s.loc, ctx->s.scal + 4, stop);
}

void launch_inv_sqrt(fosi_ctx* ctx, const double* in, double* out) {
    hipLaunchKernelGGL(k_inv_sqrt, dim3(1), dim3(64), 0, ctx->stream, in, out);
}

void launch_scale(fosi_ctx* ctx, float* x, const double* factor, int64_t n, const int* stop) {
    hipLaunchKernelGGL(k_scale, dim3(elementwise_grid(n >> 2)), dim3(kThreads), 0, ctx->stream, x, factor, n, stop);
}

void launch_diag_apply(fosi_ctx* ctx, const float* d, const float* v, float* out, int64_t n) {
    hipLaunchKernelGGL(k_diag_apply, dim3(elementwise_grid(n)), dim3(kThreads), 0, ctx->stream, d, v, out, n);
}

namespace {
// One row group of 64 rows per wave, four k-steps per register set (8 loads of 16 bytes per lane in flight), two
// workgroups per compute unit.  Measured on MI355X with 1, 2, 4 row groups, 1-4 k-steps per set and 1-4 workgroups per
// unit: everything with at least 8 loads in flight and two workgroups per unit lands within 2 % (n = 25.6 M, m = 80,
// 30 columns: 2.17-2.27 ms; n = 125 M, m = 100, 40 columns: 13.7-14.0 ms), because the kernel then runs at the rate
// the memory system gives this mix of reads and writes: a kernel with the same loads and stores and no arithmetic at
// all takes 1.9-2.2 ms on the first shape, whatever the store policy or the tile size.
template <int CB>
void ritz16_launch(fosi_ctx* ctx, const float* Q, int64_t ldq, int m, const float* S_dev, int rv, float* V, int64_t ldv,
                   int64_t n) {
    constexpr int RG = 1, U = 4;
    const int64_t ntiles = ((n >> 2) + RG * 16 - 1) / (RG * 16);
    int64_t grid = (ntiles + 3) / 4;
    const int64_t cap = (int64_t)ctx->sm_count * 2;      // resident workgroups; the kernel grid-strides over row tiles
    if (grid > cap) grid = cap;
    if (grid < 1) grid = 1;
    const size_t lds = sizeof(float) * ritz16_pitch<CB>() * ((m + 3) & ~3);
    hipLaunchKernelGGL((k_ritz_vectors_mfma16<CB, RG, U>), dim3((unsigned)grid), dim3(kThreads), lds, ctx->stream, Q, ldq, m,
                       S_dev, rv, V, ldv, n);
}
}  // namespace

// S_dev: m x (16 cb) row-major, zero padded, cb = ceil(rv / 16) <= 4
void launch_ritz_vectors_mfma(fosi_ctx* ctx, const float* Q, int64_t ldq, int m, const float* S_dev, int rv, float* V,
                              int64_t ldv, int64_t n) {
    const int cb = (rv + 15) / 16;
    if (cb <= 1) ritz16_launch<1>(ctx, Q, ldq, m, S_dev, rv, V, ldv, n);
    else if (cb == 2) ritz16_launch<2>(ctx, Q, ldq, m, S_dev, rv, V, ldv, n);
    else if (cb == 3) ritz16_launch<3>(ctx, Q, ldq, m, S_dev, rv, V, ldv, n);
    else ritz16_launch<4>(ctx, Q, ldq, m, S_dev, rv, V, ldv, n);
}

void launch_ritz_vectors(fosi_ctx* ctx, const float* Q, int64_t ldq, int m, const float* S_dev, int rv_pad, int rv,
                         float* V, int64_t ldv, int64_t n) {
    const int grid = elementwise_grid(n >> 2);
#define FOSI_RITZ(RV)                                                                                            \
    hipLaunchKernelGGL((k_ritz_vectors<RV>), dim3(grid), dim3(kThreads), 0, ctx->stream, Q, ldq, m, S_dev, rv, V, \
                       ldv, n)
    switch (rv_pad) {
        case 8: FOSI_RITZ(8); break;
        case 16: FOSI_RITZ(16); break;
        case 24: FOSI_RITZ(24); break;
        case 32: FOSI_RITZ(32); break;
        default: FOSI_RITZ(40); break;
    }
#undef FOSI_RITZ
}

void launch_step_coefficients(fosi_ctx* ctx, int rv, double lr) {
    if (rv <= 0) return;
    hipLaunchKernelGGL(k_step_coefficients, dim3((rv + 63) / 64), dim3(64), 0, ctx->stream, ctx->s.coef_a,
                       ctx->s.coef_b, ctx->s.newton, lr, rv, ctx->s.coef_c);
}

void launch_admm_begin(fosi_ctx* ctx, int64_t n, double inv_sigma, const float* pi, float* anchor, float* wa) {
    hipLaunchKernelGGL(k_admm_begin, dim3(elementwise_grid(n)), dim3(kThreads), 0, ctx->stream, n, inv_sigma, pi,
                       anchor, wa);
}

void launch_admm_end(fosi_ctx* ctx, int64_t n, double sigma, const float* anchor, const float* wa, float* pi) {
    hipLaunchKernelGGL(k_admm_end, dim3(elementwise_grid(n)), dim3(kThreads), 0, ctx->stream, n, sigma, anchor, wa,
                       pi);
}

void launch_complement_reproject(fosi_ctx* ctx, int opt, const float* V, int64_t ldv, int rv, const double* c,
                                 const float* g, const float* pi, const float* w, float* m, float* v, float* o_out,
                                 int64_t n, double mu, double b1, double b2, double inv_bc1, double inv_bc2, double eps,
                                 double lr, double wd, double* e_out, int prof_cls, double prof_bytes) {
    // columns per wave: at most 16 up to 32 columns, 24 up to 192 (a 40-column basis then splits 20 + 20 over two
    // waves instead of 14 + 14 + 12 over three: one exchange partner less per tile), 32 beyond; no empty wave
    int per_wave = ctx->tun.step_cols_per_wave;
    if (per_wave != 16 && per_wave != 24 && per_wave != 32) per_wave = rv <= 32 ? 16 : rv <= 192 ? 24 : 32;
    // the AdamW variant carries two more state vectors per row and does not fit 24 columns in registers
    if (opt == 1 && ctx->tun.step_cols_per_wave == 0 && rv <= 128) per_wave = 16;
    int S = (rv + per_wave - 1) / per_wave;
    if (S < 1) S = 1;
    if (S > 8) S = 8;
    const int cw = rv > 0 ? (rv + S - 1) / S : 1;
    S = rv > 0 ? (rv + cw - 1) / cw : 1;
    const int64_t ntiles = ((n >> 2) + 63) >> 6;
    // a whole number of blocks per compute unit: the blocks stride over the tiles in lockstep, so a unit that holds
    // one block more than its neighbours finishes that much later
    int64_t per_cu = ctx->tun.step_waves_per_cu / S;
    if (per_cu < 1) per_cu = 1;
    int64_t blocks = (int64_t)ctx->sm_count * per_cu;
    if (blocks > kMaxDotSlots) blocks = kMaxDotSlots;
    if (blocks > ntiles) blocks = ntiles;
    if (blocks < 1) blocks = 1;
    const size_t lds = S > 1 ? sizeof(double) * 2 * S * 4 * 64 : 0;
    OptScalars p{mu, b1, b2, inv_bc1, inv_bc2, eps, lr, wd};
    if (prof_cls >= 0) prof_begin(ctx, prof_cls, prof_bytes);
#define FOSI_CR(NCOL)                                                                                              \
    do {                                                                                                           \
        if (opt == 0)                                                                                              \
            hipLaunchKernelGGL((k_complement_reproject<0, NCOL>), dim3((unsigned)blocks), dim3(64 * S), lds,        \
                               ctx->stream, V, ldv, rv, cw, c, g, pi, w, m, v, o_out, n, p, ctx->s.partials);      \
        else                                                                                                       \
            hipLaunchKernelGGL((k_complement_reproject<1, NCOL>), dim3((unsigned)blocks), dim3(64 * S), lds,        \
                               ctx->stream, V, ldv, rv, cw, c, g, pi, w, m, v, o_out, n, p, ctx->s.partials);      \
    } while (0)
    if (cw <= 4) FOSI_CR(4);
    else if (cw <= 8) FOSI_CR(8);
    else if (cw <= 12) FOSI_CR(12);
    else if (cw <= 16) FOSI_CR(16);
    else if (cw <= 20) FOSI_CR(20);
    else if (cw <= 24) FOSI_CR(24);
    else FOSI_CR(32);
#undef FOSI_CR
    if (prof_cls >= 0) prof_end(ctx);
    if (rv > 0)
        hipLaunchKernelGGL(k_reduce_columns, dim3(rv + 1), dim3(64), 0, ctx->stream, ctx->s.partials, (int)blocks, (int64_t)1,
                           (int64_t)blocks, e_out, (const float*)nullptr, 0, 1.0, rv, (const double*)nullptr,
                           (const int*)nullptr, make_tail(ctx, 0, 0, 0.0));
}

void launch_step_coefficients_plus(fosi_ctx* ctx, int rv) {
    if (rv <= 0) return;
    hipLaunchKernelGGL(k_step_coefficients_plus, dim3((rv + 63) / 64), dim3(64), 0, ctx->stream, ctx->s.coef_a,
                       ctx->s.coef_b, ctx->s.newton, rv, ctx->s.coef_c);
}

/* --------------------------------------------------------------- memory-only model of a sweep (measurement aid) */
namespace {

// Reads cols_in columns of A and writes cols_out columns of B with the loads, the stores and the tiling of the
// sweeps above (a workgroup owns RPT * 1024 consecutive rows, CU columns of loads in flight per thread) and no
// arithmetic beyond one add per loaded value: what it reaches is what the memory system gives to that mix of
// reads and writes.  Column w of B receives (w + 1) * (sum of the columns of A); with cols_in == 0 the sum is 0.
template <int RPT, int CU>
__global__ __launch_bounds__(kThreads) void k_traffic_model(const float* __restrict__ A, int64_t lda, int cols_in,
                                                            float* __restrict__ Bm, int64_t ldb, int cols_out,
                                                            int64_t n4) {
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)blockIdx.x * (RPT * kThreads);
    int64_t r4[RPT];                      // float4 row group of each slot; slots past the end repeat the last group
#pragma unroll
    for (int q = 0; q < RPT; ++q) {
        r4[q] = base + q * kThreads + tid;
        if (r4[q] >= n4) r4[q] = n4 - 1;
    }
    float4 s[RPT];
#pragma unroll
    for (int q = 0; q < RPT; ++q) s[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    int j = 0;
    for (; j + CU <= cols_in; j += CU) {
        float4 a[CU][RPT];
#pragma unroll
        for (int u = 0; u < CU; ++u)
#pragma unroll
            for (int q = 0; q < RPT; ++q) a[u][q] = load_stream4(A + (int64_t)(j + u) * lda + (r4[q] << 2));
#pragma unroll
        for (int u = 0; u < CU; ++u)
#pragma unroll
            for (int q = 0; q < RPT; ++q) {
                s[q].x += a[u][q].x; s[q].y += a[u][q].y; s[q].z += a[u][q].z; s[q].w += a[u][q].w;
            }
    }
    for (; j < cols_in; ++j)
#pragma unroll
        for (int q = 0; q < RPT; ++q) {
            const float4 a = load_stream4(A + (int64_t)j * lda + (r4[q] << 2));
            s[q].x += a.x; s[q].y += a.y; s[q].z += a.z; s[q].w += a.w;
        }
    for (int w = 0; w < cols_out; ++w) {
        const float f = (float)(w + 1);
#pragma unroll
        for (int q = 0; q < RPT; ++q)
            store_stream4(Bm + (int64_t)w * ldb + (r4[q] << 2), make_float4(f * s[q].x, f * s[q].y, f * s[q].z, f * s[q].w));
    }
    // keeps the loads alive when nothing is stored (the condition never holds for finite data)
    if (cols_out == 0 && s[0].x != s[0].x && Bm != nullptr) Bm[0] = s[0].x;
}

}  // namespace

// n is a multiple of 4 (whole 16-byte row groups); large_tiles selects the launch shape the library uses above 8 M rows
void launch_traffic_model(fosi_ctx* ctx, const float* A, int64_t lda, int cols_in, float* Bm, int64_t ldb, int cols_out,
                          int64_t n, bool large_tiles) {
    const int64_t n4 = n >> 2;
    if (large_tiles) {
        const int64_t tiles = (n4 + 8 * kThreads - 1) / (8 * kThreads);
        hipLaunchKernelGGL((k_traffic_model<8, 4>), dim3((unsigned)tiles), dim3(kThreads), 0, ctx->stream, A, lda, cols_in,
                           Bm, ldb, cols_out, n4);
    } else {
        const int64_t tiles = (n4 + 4 * kThreads - 1) / (4 * kThreads);
        hipLaunchKernelGGL((k_traffic_model<4, 8>), dim3((unsigned)tiles), dim3(kThreads), 0, ctx->stream, A, lda, cols_in,
                           Bm, ldb, cols_out, n4);
    }
}


}  // namespace fosi
