// Softmax-classifier generalised Gauss-Newton operator
//     H v = X^T [ (diag(p_b) - p_b p_b^T) (X V)_b ]_b / B ,   V = v viewed as d x C row-major,
// the one dense contraction on the path: two fp32 GEMMs on the matrix cores
// (v_mfma_f32_32x32x2_f32, 64-lane wavefronts) around a row-wise
// softmax-Jacobian.  The shapes are small (B x d x C = 512 x 2048 x 1000 in the
// reference workload: 2 x 2.1 GFLOP), so the first GEMM is split along K to
// give every CU a tile; the partial products are summed inside the
// softmax-Jacobian kernel, in a fixed order.  Both products take their A operand
// k-major (K x M): the second one reads X as it is (k = batch index), the first
// one a transposed copy of X made once per operator, so that every tile is a set
// of whole 16-byte groups along its rows.  Three kernels for the products: tiles
// loaded from global memory straight into LDS (k_gemm_f32_direct; whole K-steps),
// tiles staged through registers with masks (k_gemm_f32_aligned; any K), and a
// scalar one for shapes that are not multiples of 4 (k_gemm_f32).
#include "fosi_internal.h"

namespace fosi {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Tile of a workgroup.  The hardware hands workgroups to the 8 XCDs round-robin (linear id mod 8) and each XCD
// has an L2 of its own, so with the natural (x, y, z) mapping every XCD ends up touching all of A and all of B
// and neither stays in its L2: at 8192 x 2048 x 1000 the product then pulls ~770 MB through the fabric for 40 MB
// of operands and is bound by that traffic, not by the matrix cores.  Here XCD x takes a contiguous range of the
// tile sequence (n fastest, then m, then the K split): the tiles that share a row block of A run on the same
// XCD at the same time and the XCD's share of A is fetched once.  Launch ceil(T / 8) * 8 workgroups in one
// dimension; returns false for the padding workgroups.
__device__ __forceinline__ bool xcd_tile(int gn, int gm, int gz, int& tn, int& tm, int& tz) {
    const int T = gn * gm * gz, per = (T + 7) / 8;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int t = xcd * per + slot;
    if (slot >= per || t >= T) return false;
    tn = t % gn;
    tm = (t / gn) % gm;
    tz = t / (gn * gm);
    return true;
}

// Workgroup barrier for LDS hand-over inside the K loops.  __syncthreads() also waits for every outstanding
// global load (vmcnt(0)), which would make the register lookahead of the loops below pointless: each K-step
// would again pay a full memory round trip.  Here only LDS traffic is drained; the global loads in flight
// target registers that no other wave touches.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

constexpr int TM = 64, TN = 64;            // workgroup tile; each of the 4 waves owns a 32 x 32 quadrant
constexpr int TK = 16;                     // K-step of the generic kernel
constexpr int FK = 32;                     // K-step of the aligned-shape kernel (plans use multiples of FK)
constexpr int LDT = TM;                    // LDS rows are written and read as whole 16-byte groups: no padding needed

// C[z] (M x N, row-major, ldc) = scale * A^T[:, kz] * B[kz, :]   over the K range of split z.
// A is given k-major (K x M row-major, lda), B is K x N row-major.  VEC: every row start and every 4-column
// group is 16-byte aligned.
template <bool VEC>
__global__ __launch_bounds__(256) void k_gemm_f32(const float* __restrict__ A, int lda, const float* __restrict__ Bm,
                                                  int ldb, float* __restrict__ Cout, int ldc, int M, int N, int K,
                                                  int klen, int nsplit, int64_t cstride, float scale) {
    __shared__ float As[2][TK][LDT];   // [k][m]
    __shared__ float Bs[2][TK][LDT];   // [k][n]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32;
    int tn, tm, tz;
    if (!xcd_tile((N + TN - 1) / TN, (M + TM - 1) / TM, nsplit, tn, tm, tz)) return;
    const int m0 = tm * TM, n0 = tn * TN;
    const int kbeg = tz * klen;
    const int kend = min(K, kbeg + klen);

    // this thread's slots in the two tiles
    const int bk = tid >> 4, bn4 = (tid & 15) * 4;          // both tiles: row k, 4 columns
    float ra[4], rb[4];

    auto load = [&](int k0) {
        {   // B tile
            const int k = k0 + bk, n = n0 + bn4;
            const float* p = Bm + (int64_t)k * ldb + n;
            if (VEC && k < kend && n + 3 < N) {
                const float4 v = *reinterpret_cast<const float4*>(p);
                rb[0] = v.x; rb[1] = v.y; rb[2] = v.z; rb[3] = v.w;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) rb[i] = (k < kend && n + i < N) ? p[i] : 0.f;
            }
        }
        {   // A tile
            const int k = k0 + bk, m = m0 + bn4;
            const float* p = A + (int64_t)k * lda + m;
            if (VEC && k < kend && m + 3 < M) {
                const float4 v = *reinterpret_cast<const float4*>(p);
                ra[0] = v.x; ra[1] = v.y; ra[2] = v.z; ra[3] = v.w;
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) ra[i] = (k < kend && m + i < M) ? p[i] : 0.f;
            }
        }
    };
    auto store = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) Bs[buf][bk][bn4 + i] = rb[i];
#pragma unroll
        for (int i = 0; i < 4; ++i) As[buf][bk][bn4 + i] = ra[i];
    };

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;

    const int nk = (kend - kbeg + TK - 1) / TK;
    if (nk > 0) {
        load(kbeg);
        store(0);
    }
    __syncthreads();
    const int half = lane >> 5, l32 = lane & 31;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load(kbeg + (kt + 1) * TK);       // next tile into registers while this one is multiplied
#pragma unroll
        for (int kk = 0; kk < TK; kk += 2) {
            const float a = As[buf][kk + half][wm + l32];
            const float b = Bs[buf][kk + half][wn + l32];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
        if (kt + 1 < nk) store(buf ^ 1);
        lds_barrier();
    }
    float* Cz = Cout + (int64_t)tz * cstride;
    const int col = n0 + wn + l32;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm + 8 * (v >> 2) + 4 * half + (v & 3);
        if (row < M && col < N) Cz[(int64_t)row * ldc + col] = acc[v] * scale;
    }
}

// The same product for aligned shapes (all row starts 16-byte aligned, N and the contiguous extent of A
// multiples of 4): the generic kernel above keeps its loads behind bounds tests and looks one K-step of
// 16 ahead, which leaves the matrix cores waiting for memory (measured on 512 x 1000 x 2048: 43 % busy).
// Here every global load is unconditional from a clamped, always valid address, the bounds masks are
// applied when the registers are written to LDS, the K-step is 32 (16 matrix instructions per wave
// between two barriers) and the registers run FPF K-steps ahead of the LDS tiles, which are double
// buffered so that one LDS-only barrier per K-step suffices.
constexpr int FPF = 2;
typedef unsigned int uint4v_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float4 mask4(const float4 v, const unsigned int keep) {
    uint4v_t x = __builtin_bit_cast(uint4v_t, v);
    x &= keep;
    return __builtin_bit_cast(float4, x);
}

// FULLK: K and the split length are multiples of FK, so every K-step of a split is whole: the addresses then
// advance by a constant per K-step and the bounds masks do not depend on k (computed once); otherwise every load
// clamps its k index and every LDS write masks it, ~40 more vector instructions per K-step.
// WM: the workgroup tile is 64 WM rows x 64 columns, computed by 4 WM waves (32 x 32 each).  WM = 2 (512 threads, one
// workgroup per CU) shares each B tile among twice as many rows: a quarter less operand traffic through the L1 per
// flop, which is what these products wait for.
template <bool FULLK, int WM>
__global__ __launch_bounds__(256 * WM) void k_gemm_f32_aligned(const float* __restrict__ A, int lda,
                                                               const float* __restrict__ Bm, int ldb,
                                                               float* __restrict__ Cout, int ldc, int M, int N, int K,
                                                               int klen, int nsplit, int64_t cstride, float scale) {
    constexpr int TMV = TM * WM;                                    // rows of the workgroup tile
    constexpr int NB = 2 / WM;                                      // 16-byte loads per thread and K-step: B tile (A: 2)
    __shared__ __attribute__((aligned(16))) float As[2][FK][TMV];       // [k][m]
    __shared__ __attribute__((aligned(16))) float Bs[2][FK][LDT];       // [k][n]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32;
    int tn, tm, tz;
    if (!xcd_tile((N + TN - 1) / TN, (M + TMV - 1) / TMV, nsplit, tn, tm, tz)) return;
    const int m0 = tm * TMV, n0 = tn * TN;
    const int kbeg = tz * klen;
    const int kend = min(K, kbeg + klen);
    const int nk = (kend - kbeg + FK - 1) / FK;

    // both tiles are k-major.  B: rows kr + 16 WM j (j < NB), four columns from c4; A: rows kra + 16 j (j < 2),
    // four columns from c4a
    const int kr = tid >> 4, c4 = (tid & 15) * 4;
    const int kra = tid / (16 * WM), c4a = (tid % (16 * WM)) * 4;
    float4 ra[FPF][2], rb[FPF][NB];

    // k-independent parts: clamped column / row offsets and the masks of the m and n bounds
    const int nb = n0 + c4, ma = m0 + c4a;
    const unsigned int keep_n = nb < N ? 0xffffffffu : 0u;
    const unsigned int keep_mk = ma < M ? 0xffffffffu : 0u;
    const float* pB = Bm + (nb < N ? nb : 0);
    const float* pAk = A + (ma < M ? ma : 0);                                      // + k * lda

    auto load = [&](int kt, float4* qa, float4* qb) {
        if (FULLK) {
            const int k0 = kbeg + min(kt, nk - 1) * FK;      // past the end: the last K-step again (never stored)
#pragma unroll
            for (int j = 0; j < NB; ++j) qb[j] = *reinterpret_cast<const float4*>(pB + (int64_t)(k0 + kr + 16 * WM * j) * ldb);
#pragma unroll
            for (int j = 0; j < 2; ++j) qa[j] = *reinterpret_cast<const float4*>(pAk + (int64_t)(k0 + kra + 16 * j) * lda);
        } else {
            const int k0 = kbeg + kt * FK;
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int k = k0 + kr + 16 * WM * j;
                qb[j] = *reinterpret_cast<const float4*>(pB + (int64_t)(k < kend ? k : 0) * ldb);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int k = k0 + kra + 16 * j;
                qa[j] = *reinterpret_cast<const float4*>(pAk + (int64_t)(k < kend ? k : 0) * lda);
            }
        }
    };
    auto store = [&](int kt, int buf, const float4* qa, const float4* qb) {
        const int k0 = kbeg + kt * FK;
        // (FULLK: a K-step past the range, reached only through the rounded-up trip count, must store zeros too)
        const unsigned int in_range = kt < nk ? 0xffffffffu : 0u;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int kl = kr + 16 * WM * j;
            const unsigned int keep_k = FULLK ? in_range : (k0 + kl < kend ? 0xffffffffu : 0u);
            *reinterpret_cast<float4*>(&Bs[buf][kl][c4]) = mask4(qb[j], keep_k & keep_n);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int kl = kra + 16 * j;
            const unsigned int keep_k = FULLK ? in_range : (k0 + kl < kend ? 0xffffffffu : 0u);
            *reinterpret_cast<float4*>(&As[buf][kl][c4a]) = mask4(qa[j], keep_k & keep_mk);
        }
    };

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;

    const int half = lane >> 5, l32 = lane & 31;
    // (K-steps past the end of the range load clamped addresses and store zeros)
    // the fences keep the issue order of the register sets (oldest first), so that waiting for one set
    // leaves the younger one in flight, and keep the refill in front of the matrix instructions
#pragma unroll
    for (int u = 0; u < FPF; ++u) {
        load(u, ra[u], rb[u]);
        __builtin_amdgcn_sched_barrier(0);
    }
    // The trip count is rounded up to a multiple of FPF (a K-step past the range stores zeros: its masks are all
    // off), so that the unrolled body has no branch: with one, the compiler merges the paths' outstanding-load
    // counts and ends up waiting for the younger register set as well, which halves the lookahead.
    const int nk_even = (nk + FPF - 1) / FPF * FPF;
    for (int kt0 = 0; kt0 < nk_even; kt0 += FPF) {
#pragma unroll
        for (int u = 0; u < FPF; ++u) {
            const int kt = kt0 + u;
            const int buf = u & 1;                                  // FPF is even: kt and u have the same parity
            // this buffer was last read two K-steps ago, and every wave has passed the barrier of the
            // K-step in between since
            store(kt, buf, ra[u], rb[u]);
            lds_barrier();
            load(kt + FPF, ra[u], rb[u]);                           // refill the registers just consumed
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kk = 0; kk < FK; kk += 2) {
                const float a = As[buf][kk + half][wm + l32];
                const float b = Bs[buf][kk + half][wn + l32];
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
            }
        }
    }
    float* Cz = Cout + (int64_t)tz * cstride;
    const int col = n0 + wn + l32;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm + 8 * (v >> 2) + 4 * half + (v & 3);
        if (row < M && col < N) Cz[(int64_t)row * ldc + col] = acc[v] * scale;
    }
}

// The same product with the operand tiles loaded from global memory straight into LDS (global_load_lds_dwordx4:
// lane l of a wave deposits its 16 bytes at the wave's LDS base + 16 l, so a wave instruction fills 1 KiB of
// contiguous LDS -- two rows of a 128-wide tile, four rows of a 64-wide one -- and the rows are stored without
// padding).  No registers and no LDS-write instructions are spent on staging, which is what the register-staged
// kernel above waits for.  Three tiles per operand: during K-step t a wave multiplies tile t while tiles t + 1
// and t + 2 are in flight; the loads of tile t + 2 are issued behind the barrier that opens K-step t, when every
// wave has finished with tile t - 1, whose buffer they overwrite.  Only for whole K-steps (K and the split length
// multiples of FK): data lands in LDS unmasked, which is harmless along m and n (a column of A past M or of B past
// N only reaches outputs that are not stored; its address is clamped to a valid one) but not along k.
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

// Rendezvous of the workgroup with LDS-only ordering: the bare barrier intrinsic carries no memory semantics, so
// nothing would forbid the compiler to move the LDS reads of the new tile above it; the two fences do (workgroup
// scope, LDS address space only: they cost a wait for this wave's own LDS traffic, not for global memory).
__device__ __forceinline__ void tile_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int WM>
__global__ __launch_bounds__(256 * WM) void k_gemm_f32_direct(const float* __restrict__ A, int lda,
                                                              const float* __restrict__ Bm, int ldb,
                                                              float* __restrict__ Cout, int ldc, int M, int N, int K,
                                                              int klen, int nsplit, int64_t cstride, float scale) {
    constexpr int TMV = TM * WM, NW = 4 * WM;
    constexpr int A_RPI = 256 / TMV, B_RPI = 256 / TN;              // tile rows filled by one wave instruction (1 KiB)
    constexpr int A_IPW = FK / A_RPI / NW, B_IPW = FK / B_RPI / NW; // instructions per wave and tile
    __shared__ __attribute__((aligned(16))) float As0[FK][TMV], As1[FK][TMV], As2[FK][TMV];   // [k][m]
    __shared__ __attribute__((aligned(16))) float Bs0[FK][TN], Bs1[FK][TN], Bs2[FK][TN];      // [k][n]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32;
    int tn, tm, tz;
    if (!xcd_tile((N + TN - 1) / TN, (M + TMV - 1) / TMV, nsplit, tn, tm, tz)) return;
    const int m0 = tm * TMV, n0 = tn * TN;
    const int kbeg = tz * klen;
    const int nk = (min(K, kbeg + klen) - kbeg) / FK;

    // this lane's source of every load: row offset inside a wave instruction and clamped column
    const int a_row = lane / (TMV / 4), a_col = m0 + (lane % (TMV / 4)) * 4;
    const int b_row = lane / (TN / 4), b_col = n0 + (lane % (TN / 4)) * 4;
    const int64_t oA = (a_col < M ? a_col : 0) + (int64_t)(kbeg + a_row) * lda;      // float offsets of this lane
    const int64_t oB = (b_col < N ? b_col : 0) + (int64_t)(kbeg + b_row) * ldb;

    auto issue = [&](int kt, float (*As)[TMV], float (*Bs)[TN]) {
#pragma unroll
        for (int i = 0; i < A_IPW; ++i) {
            const int r = (wave + NW * i) * A_RPI;                  // first tile row of this instruction (uniform)
            __builtin_amdgcn_global_load_lds((glb_ptr_t)(A + oA + (int64_t)(kt * FK + r) * lda), (lds_ptr_t)&As[r][0], 16, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < B_IPW; ++i) {
            const int r = (wave + NW * i) * B_RPI;
            __builtin_amdgcn_global_load_lds((glb_ptr_t)(Bm + oB + (int64_t)(kt * FK + r) * ldb), (lds_ptr_t)&Bs[r][0], 16, 0, 0);
        }
    };

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const int half = lane >> 5, l32 = lane & 31;
    float av[FK / 2], bv[FK / 2];                                   // a K-step's operands of this lane
    auto fetch = [&](const float (*As)[TMV], const float (*Bs)[TN]) {
#pragma unroll
        for (int i = 0; i < FK / 2; ++i) {
            av[i] = As[2 * i + half][wm + l32];
            bv[i] = Bs[2 * i + half][wn + l32];
        }
    };
    auto multiply = [&]() {
#pragma unroll
        for (int i = 0; i < FK / 2; ++i) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[i], acc, 0, 0, 0);
    };
    // vmcnt(n) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, the other counters left at their maxima)
    constexpr int LPT = A_IPW + B_IPW;                              // loads per wave and tile
    constexpr int kWaitOneTileLeft = 0x0F70 | LPT, kWaitAll = 0x0F70;

    issue(0, As0, Bs0);
    if (nk > 1) issue(1, As1, Bs1);
    // one K-step: wait for this wave's part of tile kt (the explicit count is what correctness needs: the younger
    // tile may stay in flight; today's compiler, which knows that these loads write LDS, makes the release fence of
    // the barrier wait for all of them, which measures the same), meet the other waves (their parts have landed
    // too, and they are done with tile kt - 1), request this lane's operands from LDS, refill tile kt - 1's buffer,
    // multiply.  The LDS reads are issued before the refill on purpose: the compiler makes an LDS read wait for
    // every direct-to-LDS load it cannot tell apart from the read's own tile, and that is harmless here, where the
    // only loads in flight are at least a K-step old.
#define FOSI_KSTEP(kt, Ac, Bc, Ar, Br)                                                       \
    do {                                                                                     \
        if ((kt) + 1 < nk) __builtin_amdgcn_s_waitcnt(kWaitOneTileLeft);                     \
        else __builtin_amdgcn_s_waitcnt(kWaitAll);                                           \
        tile_barrier();                                                                      \
        fetch(Ac, Bc);                                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                   \
        if ((kt) + 2 < nk) issue((kt) + 2, Ar, Br);                                          \
        __builtin_amdgcn_sched_barrier(0);                                                   \
        multiply();                                                                          \
    } while (0)
    for (int kt = 0; kt < nk; kt += 3) {
        FOSI_KSTEP(kt, As0, Bs0, As2, Bs2);
        if (kt + 1 < nk) FOSI_KSTEP(kt + 1, As1, Bs1, As0, Bs0);
        if (kt + 2 < nk) FOSI_KSTEP(kt + 2, As2, Bs2, As1, Bs1);
    }
#undef FOSI_KSTEP
    float* Cz = Cout + (int64_t)tz * cstride;
    const int col = n0 + wn + l32;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm + 8 * (v >> 2) + 4 * half + (v & 3);
        if (row < M && col < N) Cz[(int64_t)row * ldc + col] = acc[v] * scale;
    }
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_down(v, off, 64));
    return v;
}
__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}
__device__ __forceinline__ double block_sum_d(double v, double* red) {
    v = wave_sum_d(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// P[b, :] = softmax(sum_s parts[s][b, :]); one workgroup per row.
__global__ __launch_bounds__(256) void k_row_softmax(const float* __restrict__ parts, int nsplit, int64_t pstride,
                                                     int C, float* __restrict__ P) {
    __shared__ float redf[4];
    __shared__ double red[4];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int64_t base = (int64_t)b * C;
    float mx = -INFINITY;
    for (int c = tid; c < C; c += 256) {
        float z = 0.f;
        for (int s = 0; s < nsplit; ++s) z += parts[s * pstride + base + c];
        mx = fmaxf(mx, z);
    }
    mx = wave_max(mx);
    if ((tid & 63) == 0) redf[tid >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(redf[0], redf[1]), fmaxf(redf[2], redf[3]));
    double sum = 0.0;
    for (int c = tid; c < C; c += 256) {
        float z = 0.f;
        for (int s = 0; s < nsplit; ++s) z += parts[s * pstride + base + c];
        sum += exp((double)z - (double)mx);
    }
    sum = block_sum_d(sum, red);
    for (int c = tid; c < C; c += 256) {
        float z = 0.f;
        for (int s = 0; s < nsplit; ++s) z += parts[s * pstride + base + c];
        P[base + c] = (float)(exp((double)z - (double)mx) / sum);
    }
}

// Row-wise softmax Jacobian: z = sum_s parts[s][b,:];  y = p . z - p (p^T z), written over parts[0][b,:].
__global__ __launch_bounds__(256) void k_softmax_jacobian(float* __restrict__ parts, int nsplit, int64_t pstride,
                                                          int C, const float* __restrict__ P) {
    __shared__ double red[4];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int64_t base = (int64_t)b * C;
    double dot = 0.0;
    for (int c = tid; c < C; c += 256) {
        float z = 0.f;
        for (int s = 0; s < nsplit; ++s) z += parts[s * pstride + base + c];
        dot = fma((double)P[base + c], (double)z, dot);
    }
    dot = block_sum_d(dot, red);
    for (int c = tid; c < C; c += 256) {
        float z = 0.f;
        for (int s = 0; s < nsplit; ++s) z += parts[s * pstride + base + c];
        const double p = P[base + c];
        parts[base + c] = (float)(p * ((double)z - dot));
    }
}

// The same for C <= 256 * ZPT: a thread keeps its ZPT entries of the row in registers, so the partial products
// and p are read once and all loads of a row are in flight together (one memory round trip, then the row sum,
// then the stores) instead of two dependent passes over the row.
template <int ZPT>
__global__ __launch_bounds__(256) void k_softmax_jacobian_reg(float* __restrict__ parts, int nsplit, int64_t pstride,
                                                              int C, const float* __restrict__ P) {
    __shared__ double red[4];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int64_t base = (int64_t)b * C;
    float z[ZPT], pv[ZPT];
#pragma unroll
    for (int i = 0; i < ZPT; ++i) {
        const int c = tid + 256 * i;
        const int cc = c < C ? c : C - 1;                 // clamped: no branch around the loads
        pv[i] = P[base + cc];
        float acc = 0.f;
        for (int s = 0; s < nsplit; ++s) acc += parts[s * pstride + base + cc];
        z[i] = acc;
    }
    double dot = 0.0;
#pragma unroll
    for (int i = 0; i < ZPT; ++i)
        if (tid + 256 * i < C) dot = fma((double)pv[i], (double)z[i], dot);
    dot = block_sum_d(dot, red);
#pragma unroll
    for (int i = 0; i < ZPT; ++i) {
        const int c = tid + 256 * i;
        if (c < C) parts[base + c] = (float)((double)pv[i] * ((double)z[i] - dot));
    }
}

void launch_softmax_jacobian(fosi_ctx* ctx, float* parts, int nsplit, int64_t pstride, int B, int C, const float* P) {
    if (C <= 1024)
        hipLaunchKernelGGL((k_softmax_jacobian_reg<4>), dim3(B), dim3(256), 0, ctx->stream, parts, nsplit, pstride, C, P);
    else if (C <= 2048)
        hipLaunchKernelGGL((k_softmax_jacobian_reg<8>), dim3(B), dim3(256), 0, ctx->stream, parts, nsplit, pstride, C, P);
    else
        hipLaunchKernelGGL(k_softmax_jacobian, dim3(B), dim3(256), 0, ctx->stream, parts, nsplit, pstride, C, P);
}

// ---------------------------------------------------------------- bf16 matrix cores, split operand
// C[z] (M x N, row-major, ldc) = A[:, kz] * B[kz, :] with A given in bf16 (M x K row-major, k
// contiguous) and the fp32 matrix B (K x N) given as two bf16 matrices, b = hi + lo with
// |b - hi - lo| <= 2^-18 |b| (k_split_transpose), both stored transposed (N x K, k contiguous).  Both
// parts go through v_mfma_f32_32x32x16_bf16 with fp32 accumulation: the data matrix is exact in bf16,
// the vector operand keeps ~17 bits, at twice the bf16 cost instead of the 16x more expensive fp32
// matrix path.  Workgroup tile 128 x 128, K-step 64, one set of LDS tiles (two barriers per K-step); the
// four waves own 64 x 64 quadrants (2 x 2 MFMA tiles).  Operand layout of the instruction (checked against a host product): lane l supplies, for
// A, row l % 32 and the 8 consecutive k values starting at 8 (l / 32); for B, column l % 32 and the
// same k values; so all three tiles sit in LDS with k contiguous, are staged with 16-byte copies and
// fetched with 16-byte reads.
// What was measured on the way (batch 8192 x 2048 x 1000, per product of 33.5 GFLOP): splitting B
// inside this kernel while staging it costs ~300 vector instructions per wave and K-step, more than
// the 16 matrix instructions take (114 us); selects on loaded values let the compiler put every load
// under a branch that ends in a full wait, eight memory round trips per K-step (114 us as well, with
// either variant of the split) -- hence the split in a kernel of its own, unconditional loads with
// clamped addresses, masks applied when the registers are consumed, and PF K-steps of lookahead.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short ushort8 __attribute__((ext_vector_type(8)));

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDK = BK + 8;    // LDS row stride in bf16 (144 bytes: an odd number of 16-byte units, conflict-free reads)
constexpr int PF = 2;          // K-steps of register lookahead for the global loads

__device__ __forceinline__ unsigned short bf16_round(float f) {      // round to nearest even; finite inputs
    unsigned int u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
__device__ __forceinline__ float bf16_value(unsigned short h) { return __uint_as_float((unsigned int)h << 16); }

// hi_t[n, k], lo_t[n, k] (N x K, leading dimension ldt) from src[k, n] (K x N row-major, leading dimension lds_).
__global__ __launch_bounds__(256) void k_split_transpose(const float* __restrict__ src, int K, int N, int lds_,
                                                         unsigned short* __restrict__ hi_t,
                                                         unsigned short* __restrict__ lo_t, int ldt) {
    __shared__ unsigned short th[32][33], tl[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
    const int n0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
    for (int i = ty; i < 32; i += 8) {
        const int k = k0 + i, n = n0 + tx;
        float v = 0.f;
        if (k < K && n < N) v = src[(int64_t)k * lds_ + n];
        const unsigned short hi = bf16_round(v);
        th[i][tx] = hi;
        tl[i][tx] = bf16_round(v - bf16_value(hi));
    }
    __syncthreads();
    for (int i = ty; i < 32; i += 8) {
        const int n = n0 + i, k = k0 + tx;
        if (n < N && k < K) {
            hi_t[(int64_t)n * ldt + k] = th[tx][i];
            lo_t[(int64_t)n * ldt + k] = tl[tx][i];
        }
    }
}

// VEC: all three matrices have 16-byte aligned rows and K is a multiple of 8 (an 8-value chunk then lies
// inside the K range of the split or outside it).
template <bool VEC>
__global__ __launch_bounds__(256, 2) void k_gemm_bf16x2(const unsigned short* __restrict__ A, int lda,
                                                     const unsigned short* __restrict__ Bht,
                                                     const unsigned short* __restrict__ Blt, int ldbt,
                                                     float* __restrict__ Cout, int ldc, int M, int N, int K, int klen,
                                                     int nsplit, int64_t cstride, float scale) {
    __shared__ __attribute__((aligned(16))) unsigned short As[BM][LDK];
    __shared__ __attribute__((aligned(16))) unsigned short Bh[BN][LDK];
    __shared__ __attribute__((aligned(16))) unsigned short Bl[BN][LDK];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    int tn, tm, tz;
    if (!xcd_tile((N + BN - 1) / BN, (M + BM - 1) / BM, nsplit, tn, tm, tz)) return;
    const int m0 = tm * BM, n0 = tn * BN;
    const int kbeg = tz * klen;
    const int kend = min(K, kbeg + klen);

    // staging: 8 consecutive lanes cover the 128 bytes (64 k values) of one tile row, so a wave instruction
    // touches 8 cache lines (not 32) and writes LDS without bank conflicts; a thread owns the 16-byte chunk
    // sc of rows sr, sr + 32, sr + 64, sr + 96 in each of the three tiles.
    const int sc = (tid & 7) * 8, sr = tid >> 3;
    ushort8 r[PF][12];

    // raw loads from clamped (always valid) addresses; the masks are applied in store(), when the registers
    // are consumed, so that nothing here waits for memory
    auto load = [&](int k0, ushort8* q) {
        const int k = k0 + sc;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = sr + 32 * j;
            const unsigned short* pa = A + (int64_t)min(m0 + row, M - 1) * lda;
            const unsigned short* ph = Bht + (int64_t)min(n0 + row, N - 1) * ldbt;
            const unsigned short* pl = Blt + (int64_t)min(n0 + row, N - 1) * ldbt;
            if (VEC) {
                const int kc = k < kend ? k : 0;
                q[j] = *reinterpret_cast<const ushort8*>(pa + kc);
                q[4 + j] = *reinterpret_cast<const ushort8*>(ph + kc);
                q[8 + j] = *reinterpret_cast<const ushort8*>(pl + kc);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int kc = min(k + i, K - 1);
                    q[j][i] = pa[kc];
                    q[4 + j][i] = ph[kc];
                    q[8 + j][i] = pl[kc];
                }
            }
        }
    };
    auto store = [&](int k0, const ushort8* q) {
        const int k = k0 + sc;
        typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int row = sr + 32 * j;
            ushort8 t[3];
            if (VEC) {     // one mask per chunk: four dword ANDs per vector
                const unsigned int keep_a = (m0 + row < M && k < kend) ? 0xffffffffu : 0u;
                const unsigned int keep_b = (n0 + row < N && k < kend) ? 0xffffffffu : 0u;
#pragma unroll
                for (int w = 0; w < 3; ++w) {
                    uint4v x = __builtin_bit_cast(uint4v, q[4 * w + j]);
                    x &= (w == 0 ? keep_a : keep_b);
                    t[w] = __builtin_bit_cast(ushort8, x);
                }
            } else {
#pragma unroll
                for (int w = 0; w < 3; ++w)
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const bool ok = (w == 0 ? m0 + row < M : n0 + row < N) && k + i < kend;
                        t[w][i] = q[4 * w + j][i] & (ok ? (unsigned short)0xffff : (unsigned short)0);
                    }
            }
            *reinterpret_cast<ushort8*>(&As[row][sc]) = t[0];
            *reinterpret_cast<ushort8*>(&Bh[row][sc]) = t[1];
            *reinterpret_cast<ushort8*>(&Bl[row][sc]) = t[2];
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = (kend - kbeg + BK - 1) / BK;
    // (steps past the end of the K range load clamped addresses and are never stored)
#pragma unroll
    for (int u = 0; u < PF; ++u) load(kbeg + u * BK, r[u]);
    for (int kt0 = 0; kt0 < nk; kt0 += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int kt = kt0 + u;
            if (kt < nk) {                                     // uniform
                if (kt > 0) lds_barrier();                     // every wave has finished reading the previous tiles
                store(kbeg + kt * BK, r[u]);
                lds_barrier();
                load(kbeg + (kt + PF) * BK, r[u]);             // refill the registers just consumed
#pragma unroll
                for (int ks = 0; ks < BK; ks += 16) {
                    bf16x8 a[2], bh[2], bl[2];
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        a[i] = *reinterpret_cast<const bf16x8*>(&As[wm + 32 * i + l32][ks + 8 * half]);
                        bh[i] = *reinterpret_cast<const bf16x8*>(&Bh[wn + 32 * i + l32][ks + 8 * half]);
                        bl[i] = *reinterpret_cast<const bf16x8*>(&Bl[wn + 32 * i + l32][ks + 8 * half]);
                    }
                    // the small parts first; four independent accumulators between the two uses of each one
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bl[j], acc[i][j], 0, 0, 0);
#pragma unroll
                    for (int i = 0; i < 2; ++i)
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bh[j], acc[i][j], 0, 0, 0);
                }
            }
        }
    }
    float* Cz = Cout + (int64_t)tz * cstride;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn + 32 * j + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * half + (v & 3);
                if (row < M && col < N) Cz[(int64_t)row * ldc + col] = acc[i][j][v] * scale;
            }
        }
}

// XT[j, i] = X[i, j] for a bf16 matrix (rows x cols row-major -> cols x rows row-major), once per operator.
__global__ __launch_bounds__(256) void k_transpose_u16(const unsigned short* __restrict__ X, int rows, int cols,
                                                       unsigned short* __restrict__ XT) {
    __shared__ unsigned short tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = X[(int64_t)(r0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < cols && r0 + tx < rows) XT[(int64_t)(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

// XT[j, i] = X[i, j] for an fp32 matrix (rows x cols row-major -> cols x ldt row-major, ldt >= rows), once per operator.
__global__ __launch_bounds__(256) void k_transpose_f32(const float* __restrict__ X, int rows, int cols,
                                                       float* __restrict__ XT, int ldt) {
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = X[(int64_t)(r0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < cols && r0 + tx < rows) XT[(int64_t)(c0 + i) * ldt + r0 + tx] = tile[tx][i];
}

// out[i] = scale * sum_s parts[s][i]  (fixed order)
__global__ __launch_bounds__(256) void k_sum_splits(const float* __restrict__ parts, int nsplit, int64_t pstride,
                                                    int64_t count, float scale, float* __restrict__ out) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += stride) {
        float z = 0.f;
        for (int s = 0; s < nsplit; ++s) z += parts[s * pstride + i];
        out[i] = z * scale;
    }
}

struct GemmPlan {
    int nsplit, klen;
    int wm = 1;          // row-tile multiple of the aligned kernel (1: 64 rows, two workgroups per CU; 2: 128 rows, one)
};

// Row-tile multiple: the tall tile shares each B tile among twice the rows (a quarter less operand traffic per flop) but
// runs as one workgroup of eight waves per CU, whose waves meet at the same barriers; two 64 x 64 workgroups per CU
// drift apart and cover each other's barriers and LDS latencies.  Measured on d x C = 2048 x 1000 (whole operator):
// batch 512: 57.9 us with 64 x 64 tiles against 59.0 us; 2048: 164 against 173 us; 8192: 673 against 656 us -- the tall
// tile pays once there are several rounds of workgroups per CU.
int tile_rows_multiple(int M, int N, int sm_count) {
    const int tiles64 = ((M + TM - 1) / TM) * ((N + TN - 1) / TN);
    return (M >= 2 * TM && tiles64 >= 8 * sm_count) ? 2 : 1;
}

GemmPlan plan_split(int M, int N, int K, int sm_count) {
    const int wm = tile_rows_multiple(M, N, sm_count);
    const int tiles = ((M + TM * wm - 1) / (TM * wm)) * ((N + TN - 1) / TN);
    int s = (2 / wm * sm_count) / (tiles > 0 ? tiles : 1);
    if (s < 1) s = 1;
    if (s > 8) s = 8;
    int klen = ((K + s - 1) / s + FK - 1) / FK * FK;
    if (klen < FK) klen = FK;
    s = (K + klen - 1) / klen;
    return {s, klen, wm};
}

void launch_gemm(fosi_ctx* ctx, const float* A, int lda, const float* Bm, int ldb, float* Cout, int ldc, int M, int N,
                 int K, GemmPlan plan, int64_t cstride, float scale) {
    const int tiles = ((N + TN - 1) / TN) * ((M + TM - 1) / TM) * plan.nsplit;
    const dim3 grid((tiles + 7) / 8 * 8);
    const int tiles_tall = ((N + TN - 1) / TN) * ((M + 2 * TM - 1) / (2 * TM)) * plan.nsplit;
    const dim3 grid_tall((tiles_tall + 7) / 8 * 8);
    const bool vec = (lda % 4 == 0) && (ldb % 4 == 0) && ((reinterpret_cast<uintptr_t>(A) & 15) == 0) &&
                     ((reinterpret_cast<uintptr_t>(Bm) & 15) == 0);
    // whole 16-byte groups only: N (columns of B) and the contiguous extent of A (M if stored K x M, else K)
    const bool aligned = vec && N % 4 == 0 && M % 4 == 0 && plan.klen % FK == 0;
    if (aligned && K % FK == 0 && plan.wm == 2 && ctx->tun.ggn_direct)
        hipLaunchKernelGGL((k_gemm_f32_direct<2>), grid_tall, dim3(512), 0, ctx->stream, A, lda, Bm, ldb, Cout, ldc,
                           M, N, K, plan.klen, plan.nsplit, cstride, scale);
    else if (aligned && K % FK == 0 && plan.wm == 1 && ctx->tun.ggn_direct)
        hipLaunchKernelGGL((k_gemm_f32_direct<1>), grid, dim3(256), 0, ctx->stream, A, lda, Bm, ldb, Cout, ldc,
                           M, N, K, plan.klen, plan.nsplit, cstride, scale);
    else if (aligned && K % FK == 0 && plan.wm == 2)
        hipLaunchKernelGGL((k_gemm_f32_aligned<true, 2>), grid_tall, dim3(512), 0, ctx->stream, A, lda, Bm, ldb, Cout, ldc,
                           M, N, K, plan.klen, plan.nsplit, cstride, scale);
    else if (aligned && plan.wm == 2)
        hipLaunchKernelGGL((k_gemm_f32_aligned<false, 2>), grid_tall, dim3(512), 0, ctx->stream, A, lda, Bm, ldb, Cout, ldc,
                           M, N, K, plan.klen, plan.nsplit, cstride, scale);
    else if (aligned && K % FK == 0)
        hipLaunchKernelGGL((k_gemm_f32_aligned<true, 1>), grid, dim3(256), 0, ctx->stream, A, lda, Bm, ldb, Cout, ldc, M,
                           N, K, plan.klen, plan.nsplit, cstride, scale);
    else if (aligned)
        hipLaunchKernelGGL((k_gemm_f32_aligned<false, 1>), grid, dim3(256), 0, ctx->stream, A, lda, Bm, ldb, Cout, ldc, M,
                           N, K, plan.klen, plan.nsplit, cstride, scale);
    else if (vec)
        hipLaunchKernelGGL((k_gemm_f32<true>), grid, dim3(256), 0, ctx->stream, A, lda, Bm, ldb, Cout, ldc, M, N, K,
                           plan.klen, plan.nsplit, cstride, scale);
    else
        hipLaunchKernelGGL((k_gemm_f32<false>), grid, dim3(256), 0, ctx->stream, A, lda, Bm, ldb, Cout, ldc, M, N, K,
                           plan.klen, plan.nsplit, cstride, scale);
}

GemmPlan plan_split_bf16(int M, int N, int K, int sm_count) {
    const int tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    int s = (2 * sm_count) / (tiles > 0 ? tiles : 1);
    if (s < 1) s = 1;
    if (s > 8) s = 8;
    int klen = ((K + s - 1) / s + BK - 1) / BK * BK;
    if (klen < BK) klen = BK;
    s = (K + klen - 1) / klen;
    return {s, klen};
}

// Splits the fp32 matrix Bm (K x N row-major) into the operator's transposed bf16 pair (sh, sl: N x ldt), then
// C = A * Bm on the bf16 matrix cores.
void launch_gemm_bf16(fosi_ctx* ctx, const unsigned short* A, int lda, const float* Bm, int ldb, unsigned short* sh,
                      unsigned short* sl, float* Cout, int ldc, int M, int N, int K, GemmPlan plan, int64_t cstride,
                      float scale) {
    const int ldt = (K + 7) / 8 * 8;
    hipLaunchKernelGGL(k_split_transpose, dim3((N + 31) / 32, (K + 31) / 32), dim3(256), 0, ctx->stream, Bm, K, N, ldb, sh,
                       sl, ldt);
    const int tiles = ((N + BN - 1) / BN) * ((M + BM - 1) / BM) * plan.nsplit;
    const dim3 grid((tiles + 7) / 8 * 8);
    const bool vec = (lda % 8 == 0) && (K % 8 == 0) && (plan.klen % 8 == 0) &&
                     ((reinterpret_cast<uintptr_t>(A) & 15) == 0) && ((reinterpret_cast<uintptr_t>(sh) & 15) == 0) &&
                     ((reinterpret_cast<uintptr_t>(sl) & 15) == 0);
    if (vec)
        hipLaunchKernelGGL((k_gemm_bf16x2<true>), grid, dim3(256), 0, ctx->stream, A, lda, sh, sl, ldt, Cout, ldc, M, N, K,
                           plan.klen, plan.nsplit, cstride, scale);
    else
        hipLaunchKernelGGL((k_gemm_bf16x2<false>), grid, dim3(256), 0, ctx->stream, A, lda, sh, sl, ldt, Cout, ldc, M, N, K,
                           plan.klen, plan.nsplit, cstride, scale);
}

}  // namespace

fosi_status ggn_prepare(fosi_hvp* op) {
    fosi_ctx* ctx = op->ctx;
    const int B = op->B, d = op->dim, C = op->C;
    const size_t bc = (size_t)B * C;
    if (op->bf16) {
        const GemmPlan p1 = plan_split_bf16(B, C, d, ctx->sm_count), p2 = plan_split_bf16(d, C, B, ctx->sm_count);
        if (hipMalloc(reinterpret_cast<void**>(&op->P), bc * sizeof(float)) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&op->Z), bc * sizeof(float) * p1.nsplit) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&op->XTb), (size_t)B * d * sizeof(unsigned short)) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&op->Y2), (size_t)d * C * sizeof(float) * p2.nsplit) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&op->S1), 2 * (size_t)C * ((d + 7) / 8 * 8) * sizeof(unsigned short)) != hipSuccess ||
            hipMalloc(reinterpret_cast<void**>(&op->S2), 2 * (size_t)C * ((B + 7) / 8 * 8) * sizeof(unsigned short)) != hipSuccess)
            return fail(ctx, FOSI_ERR_NOMEM, "softmax-GGN work buffers");
        // the split kernel leaves the padding columns of a row (k in [K, ldt)) untouched: clear them once, the
        // product reads whole 16-byte chunks
        (void)hipMemsetAsync(op->S1, 0, 2 * (size_t)C * ((d + 7) / 8 * 8) * sizeof(unsigned short), ctx->stream);
        (void)hipMemsetAsync(op->S2, 0, 2 * (size_t)C * ((B + 7) / 8 * 8) * sizeof(unsigned short), ctx->stream);
        unsigned short* s1h = op->S1;
        unsigned short* s1l = op->S1 + (size_t)C * ((d + 7) / 8 * 8);
        hipLaunchKernelGGL(k_transpose_u16, dim3((d + 31) / 32, (B + 31) / 32), dim3(256), 0, ctx->stream, op->Xb, B, d,
                           op->XTb);
        // P = softmax(X W)
        launch_gemm_bf16(ctx, op->Xb, d, op->W, C, s1h, s1l, op->Z, C, B, C, d, p1, (int64_t)bc, 1.f);
        hipLaunchKernelGGL(k_row_softmax, dim3(B), dim3(256), 0, ctx->stream, op->Z, p1.nsplit, (int64_t)bc, C, op->P);
        return check_hip(ctx, hipGetLastError(), "softmax-GGN prepare");
    }
    const GemmPlan plan = plan_split(B, C, d, ctx->sm_count);
    op->ldxt = (B + 3) / 4 * 4;
    if (hipMalloc(reinterpret_cast<void**>(&op->P), bc * sizeof(float)) != hipSuccess ||
        hipMalloc(reinterpret_cast<void**>(&op->Z), bc * sizeof(float) * plan.nsplit) != hipSuccess ||
        hipMalloc(reinterpret_cast<void**>(&op->XT), (size_t)d * op->ldxt * sizeof(float)) != hipSuccess)
        return fail(ctx, FOSI_ERR_NOMEM, "softmax-GGN work buffers");
    // X is constant over the operator's life: a transposed copy lets the first product stage its A tiles k-major
    // with 16-byte LDS writes like the second one (with X itself the tile has to be transposed on the way into
    // LDS, four scalar writes per 16 bytes with four-way bank conflicts)
    if (op->ldxt != B) (void)hipMemsetAsync(op->XT, 0, (size_t)d * op->ldxt * sizeof(float), ctx->stream);
    hipLaunchKernelGGL(k_transpose_f32, dim3((d + 31) / 32, (B + 31) / 32), dim3(256), 0, ctx->stream, op->X, B, d, op->XT,
                       op->ldxt);
    // P = softmax(X W)
    launch_gemm(ctx, op->XT, op->ldxt, op->W, C, op->Z, C, B, C, d, plan, (int64_t)bc, 1.f);
    hipLaunchKernelGGL(k_row_softmax, dim3(B), dim3(256), 0, ctx->stream, op->Z, plan.nsplit, (int64_t)bc, C, op->P);
    return check_hip(ctx, hipGetLastError(), "softmax-GGN prepare");
}

fosi_status ggn_apply(fosi_hvp* op, const float* v, float* hv) {
    fosi_ctx* ctx = op->ctx;
    const int B = op->B, d = op->dim, C = op->C;
    const int64_t bc = (int64_t)B * C;
    if (op->bf16) {
        const GemmPlan p1 = plan_split_bf16(B, C, d, ctx->sm_count), p2 = plan_split_bf16(d, C, B, ctx->sm_count);
        const int64_t dc = (int64_t)d * C;
        unsigned short* s1h = op->S1;
        unsigned short* s1l = op->S1 + (size_t)C * ((d + 7) / 8 * 8);
        unsigned short* s2h = op->S2;
        unsigned short* s2l = op->S2 + (size_t)C * ((B + 7) / 8 * 8);
        // Z = X V (split along d), Y = softmax-Jacobian rows of Z, hv = X^T Y / B (split along the batch)
        launch_gemm_bf16(ctx, op->Xb, d, v, C, s1h, s1l, op->Z, C, B, C, d, p1, bc, 1.f);
        launch_softmax_jacobian(ctx, op->Z, p1.nsplit, bc, B, C, op->P);
        if (p2.nsplit == 1) {
            launch_gemm_bf16(ctx, op->XTb, B, op->Z, C, s2h, s2l, hv, C, d, C, B, p2, 0, 1.f / (float)B);
        } else {
            launch_gemm_bf16(ctx, op->XTb, B, op->Z, C, s2h, s2l, op->Y2, C, d, C, B, p2, dc, 1.f);
            int64_t g = (dc + 255) / 256;
            if (g > 4096) g = 4096;
            hipLaunchKernelGGL(k_sum_splits, dim3((unsigned)g), dim3(256), 0, ctx->stream, op->Y2, p2.nsplit, dc, dc,
                               1.f / (float)B, hv);
        }
        return FOSI_OK;
    }
    const GemmPlan plan = plan_split(B, C, d, ctx->sm_count);
    // Z = X V (split along d), Y = softmax-Jacobian rows of Z, hv = X^T Y / B
    launch_gemm(ctx, op->XT, op->ldxt, v, C, op->Z, C, B, C, d, plan, bc, 1.f);
    launch_softmax_jacobian(ctx, op->Z, plan.nsplit, bc, B, C, op->P);
    launch_gemm(ctx, op->X, d, op->Z, C, hv, C, d, C, B, GemmPlan{1, (B + FK - 1) / FK * FK, tile_rows_multiple(d, C, ctx->sm_count)}, 0,
                      1.f / (float)B);
    return FOSI_OK;
}

void ggn_release(fosi_hvp* op) {
    if (op->P != nullptr) (void)hipFree(op->P);
    if (op->Z != nullptr) (void)hipFree(op->Z);
    if (op->XTb != nullptr) (void)hipFree(op->XTb);
    if (op->XT != nullptr) (void)hipFree(op->XT);
    op->XT = nullptr;
    if (op->Y2 != nullptr) (void)hipFree(op->Y2);
    if (op->S1 != nullptr) (void)hipFree(op->S1);
    if (op->S2 != nullptr) (void)hipFree(op->S2);
    op->S1 = nullptr;
    op->S2 = nullptr;
    op->P = nullptr;
    op->Z = nullptr;
    op->XTb = nullptr;
    op->Y2 = nullptr;
}

}  // namespace fosi
