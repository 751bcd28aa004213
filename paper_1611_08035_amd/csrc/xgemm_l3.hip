// xgemm_l3.hip -- level-3 routines on top of the GEMM entry points: the
// triangular solve with many right-hand sides and the triangular product.
//
// Both are organised so that almost all of their arithmetic is GEMM: the
// triangular matrix is halved recursively, each half is handled in turn, and
// the coupling between the halves is one product with the off-diagonal block
// (depth = half the order, so the products are large).  Diagonal blocks of
// order <= NB are solved (multiplied) in a small kernel of their own.
#include "../../include/xgemm.h"
#include "../../include/xgemm_probe.h"
#include "../../include/xgemm_tuning.h"
#include "tables.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <type_traits>

namespace {

constexpr int NB = 64;        // order of the diagonal blocks solved by substitution

inline bool is_n(char t) { return t == 'N' || t == 'n'; }
inline bool is_t(char t) { return t == 'T' || t == 't' || t == 'C' || t == 'c'; }
inline int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }
constexpr int64_t DIM_MAX = 0x7fffffff;

template <typename T> struct BlockArgs {
    const T *A;      // top-left element of the diagonal block inside the stored triangular matrix
    int64_t lda;
    T *B;            // first element of the block's right-hand sides
    int64_t ldb;
    int nbk;         // order of the block, 1..NB
    int nrhs;        // number of right-hand sides
    int left;        // 1: right-hand side q is column q of B (elements B[r + q*ldb]); 0: row q (B[q + c*ldb])
    int etrans;      // the solve's matrix E has E(r,c) = A[c + r*lda] if set, A[r + c*lda] otherwise
    int stored_lower;   // which triangle of the stored matrix is referenced
    int unit;        // implicit unit diagonal
    T alpha;         // triangular product only: scalar applied to the result
};

// Diagonal-block solve E x = b by substitution, E of order nbk <= NB = 64.
// A workgroup of 4 waves brings E to unit lower-triangular form in LDS once:
// an upper-triangular E is reversed in both indices (and the right-hand sides
// with it), and every column is divided by its diagonal entry, E = E' D, so that
// E' y = b with y = D x has a unit diagonal and x = D^-1 y.  Each wave then
// solves RPW right-hand sides (4, 8 or 16, chosen by the host) at once with the rows of the system
// spread over its 64 lanes: lane r holds y_r of every right-hand side in
// registers.  Step c reads column c of E' (one LDS element per lane, zero on
// and above the diagonal), takes the pivot y_c of each right-hand side from
// lane c into scalar registers, and updates all rows below in one FMA per
// right-hand side:  y_r -= E'(r, c) y_c.
constexpr int WAVES = 4;

template <typename T> static __device__ __forceinline__ T lane_value(T v, int lane) {
    if constexpr (sizeof(T) == 8) {
        typedef int i32x2 __attribute__((ext_vector_type(2)));
        i32x2 p = __builtin_bit_cast(i32x2, v);
        p[0] = __builtin_amdgcn_readlane(p[0], lane);
        p[1] = __builtin_amdgcn_readlane(p[1], lane);
        return __builtin_bit_cast(T, p);
    } else {
        return __builtin_bit_cast(T, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
    }
}

// 16x16x4 matrix instruction of each precision as used by the block kernels below:
// lane l supplies element (l & 15, l >> 4) of the 16x4 row operand and element
// (l >> 4, l & 15) of the 4x16 column operand; register r of lane l holds element
// (drow(l, r), l & 15) of the 16x16 result.
template <typename T> struct Mma16;
template <> struct Mma16<double> {
    typedef double acc_t __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ acc_t mma(double row_op, double col_op, acc_t c) {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(row_op, col_op, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int drow(int lane, int r) { return (lane >> 4) + 4 * r; }
    static __device__ __forceinline__ double rsq(double x) { return __builtin_amdgcn_rsq(x); }
    static constexpr double TINY = 0x1p-767, BIG = 0x1p1000;   // pivots the fast route accepts
};
template <> struct Mma16<float> {
    typedef float acc_t __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ acc_t mma(float row_op, float col_op, acc_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(row_op, col_op, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int drow(int lane, int r) { return 4 * (lane >> 4) + r; }
    static __device__ __forceinline__ float rsq(float x) { return __builtin_amdgcn_rsqf(x); }
    static constexpr float TINY = 0x1p-96f, BIG = 0x1p100f;
};

// Compute units of the current device (256 on MI355X), read once per device.
inline int device_cus() {
    constexpr int MAX_DEV = 64;
    static std::atomic<int> cached[MAX_DEV];             // 0: not read yet
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return 256;
    if ((cus = cached[dev].load(std::memory_order_relaxed)) > 0) return cus;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
    cached[dev].store(cus, std::memory_order_relaxed);
    return cus;
}

// Dynamic LDS beyond 64 KiB has to be requested explicitly: once per kernel and device.
template <typename K> hipError_t allow_lds(K kernel, size_t bytes) {
    if (bytes <= 65536) return hipSuccess;
    constexpr int MAX_DEV = 64;
    static std::atomic<int> done[MAX_DEV];               // per instantiation, i.e. per kernel
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return hipErrorInvalidDevice;
    if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess) done[dev].store(1, std::memory_order_release);
    return e;
}

template <typename T, int RPW> __global__ void __launch_bounds__(64 * WAVES) trsm_block_kernel(const BlockArgs<T> a) {
    __shared__ T e_cols[NB * NB];            // E(r, c) at [c * NB + r], zero on and above the diagonal
    __shared__ T d_inv[NB];                  // 1 / E(c, c)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nbk = a.nbk;
    const bool e_lower = (a.stored_lower != 0) != (a.etrans != 0);
    const int lowr = a.stored_lower ? 1 : 0;
    constexpr int PER = NB / WAVES;

    // Every global load of the kernel is issued before the first wait: the
    // right-hand sides of this wave, this thread's share of the block, the diagonal.
    // right-hand sides q0 .. q0 + RPW - 1; lane holds element `pos` of each
    const int q0 = (blockIdx.x * WAVES + wave) * RPW;
    const int pos = lane < nbk ? (e_lower ? lane : nbk - 1 - lane) : 0;   // lanes past the order re-read element 0
    const int64_t qs = a.left ? a.ldb : 1, xs = a.left ? 1 : a.ldb;       // strides between / inside right-hand sides
    T *const xp = a.B + (int64_t)pos * xs;
    T y[RPW];
#pragma unroll
    for (int j = 0; j < RPW; ++j) {
        const int q = q0 + j < a.nrhs ? q0 + j : a.nrhs - 1;     // past the last one: a copy that is not stored
        y[j] = xp[(int64_t)q * qs];
    }
    // Thread (wave w, lane t) takes stored row t and the stored columns s = w, w + 4, ...; only the
    // referenced triangle is read, positions outside it re-read element (0, 0) and count as zero.
    T row[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int s = wave + u * WAVES;
        const int inside = (int)(lane < nbk) & (int)(s < nbk) & ((lowr & (int)(lane > s)) | ((lowr ^ 1) & (int)(lane < s)));
        const T v = a.A[(inside ? lane : 0) + (int64_t)(inside ? s : 0) * a.lda];
        row[u] = inside ? v : T(0);
    }
    const bool has_diag = tid < nbk && !a.unit;
    const T dv = a.A[has_diag ? tid + (int64_t)tid * a.lda : 0];

    // (stored row, stored column) -> (r, c) of E is one-to-one on the NB x NB square (positions
    // outside the block map to themselves), so every LDS element is written exactly once
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int s = wave + u * WAVES;
        const bool in_blk = lane < nbk && s < nbk;
        int r = a.etrans ? s : lane, c = a.etrans ? lane : s;
        if (in_blk && !e_lower) { r = nbk - 1 - r; c = nbk - 1 - c; }
        e_cols[c * NB + r] = row[u];
    }
    if (tid < NB) d_inv[tid < nbk ? (e_lower ? tid : nbk - 1 - tid) : tid] = has_diag ? T(1) / dv : T(1);
    __syncthreads();
    if (q0 >= a.nrhs) return;                                    // wave-uniform, after the last barrier

    // E = E' D with E' unit lower triangular: solve E' y = b, then x = D^-1 y
#pragma unroll
    for (int j = 0; j < RPW; ++j) y[j] = lane < nbk ? y[j] : T(0);
    T e = e_cols[lane] * d_inv[0];                               // column 0 of E'
#pragma unroll 1
    for (int c = 0; c < nbk; ++c) {
        const int cn = c + 1 < NB ? c + 1 : c;
        const T e_next = e_cols[cn * NB + lane] * d_inv[cn];
#pragma unroll
        for (int j = 0; j < RPW; ++j) y[j] -= e * lane_value(y[j], c);
        e = e_next;
    }
    const T d = d_inv[lane];
    if (lane < nbk) {
#pragma unroll
        for (int j = 0; j < RPW; ++j)
            if (q0 + j < a.nrhs) xp[(int64_t)(q0 + j) * qs] = y[j] * d;
    }
}

// The same solve for diagonal blocks of order up to WIDE = 64 * GROUPS: lane l of a
// solving wave holds rows l, l + 64, ... of the RPW (2, 4 or 8) systems of its wave
// (GROUPS values per system), and E' passes through LDS in panels of PANEL columns.
// Feeding a panel (DEPTH of them are on their way from memory at any time, each in
// registers of its own; each column is scaled by the reciprocal of its diagonal entry
// and written into one half of a double buffer in LDS while the other half is in
// use; one barrier per panel) costs about as many instructions as solving with it,
// and a lone wave issues them slowly.  With FEED > 0 the workgroup therefore has
// FEED feeding waves beside its WAVES solving waves, which shortens a solve with few
// right-hand sides by a third; with FEED == 0 every wave does both, which is the
// better use of a device that is full of workgroups anyway.
// One kernel of this kind replaces the four block solves and three coupling
// products that recursion down to order 64 would spend on a block of order 256.
constexpr int GROUPS = 4, WIDE = 64 * GROUPS, PANEL = 16;
template <typename T> constexpr size_t wide_lds_bytes() { return (2 * PANEL * WIDE + WIDE) * sizeof(T); }

template <typename T, int RPW, int DEPTH, int FEED, int SW>
__global__ void __launch_bounds__(64 * (SW + FEED)) trsm_wide_kernel(const BlockArgs<T> a) {
    static_assert(64 % PANEL == 0 && DEPTH >= 1 && (FEED > 0 || 64 * SW == WIDE), "panels do not straddle groups");
    constexpr int FT = FEED ? 64 * FEED : 64 * SW;      // feeding threads
    constexpr int EL = PANEL * WIDE / FT;               // elements of a panel per feeding thread
    static_assert(FT % WIDE == 0 && EL * FT == PANEL * WIDE, "whole columns of a panel per pass");
    extern __shared__ __align__(16) unsigned char wide_lds[];
    T *const e_pan = reinterpret_cast<T *>(wide_lds);   // two panels: E'(r, c0 + k) at [half * PANEL * WIDE + k * WIDE + r], zero on and above the diagonal
    T *const d_inv = e_pan + 2 * PANEL * WIDE;           // 1 / E(c, c)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool feeding = FEED == 0 || wave >= SW;        // wave-uniform; FEED == 0: every wave both feeds and solves
    const bool solving = FEED == 0 || wave < SW;
    const int tid = FEED == 0 ? (int)threadIdx.x : (int)threadIdx.x - 64 * SW;      // index among the feeding threads
    const int dim = a.nbk;
    const bool e_lower = (a.stored_lower != 0) != (a.etrans != 0);
    const int npan = (dim + PANEL - 1) / PANEL;

    // ---- solving waves: right-hand sides q0 .. q0 + RPW - 1; lane holds elements lane + 64 g of each
    const int q0 = (blockIdx.x * SW + (wave % SW)) * RPW;
    const int64_t qs = a.left ? a.ldb : 1, xs = a.left ? 1 : a.ldb;
    const bool live = solving && q0 < a.nrhs;
    T y[GROUPS][RPW];
    int64_t xoff[GROUPS];
    if (solving) {
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) {
            const int idx = lane + 64 * g;
            const int pos = idx < dim ? (e_lower ? idx : dim - 1 - idx) : 0;    // rows past the order re-read element 0
            xoff[g] = (int64_t)pos * xs;
#pragma unroll
            for (int j = 0; j < RPW; ++j) {
                const int q = q0 + j < a.nrhs ? q0 + j : a.nrhs - 1;           // past the last one: a copy that is not stored
                const T v = a.B[xoff[g] + (int64_t)q * qs];
                y[g][j] = idx < dim ? v : T(0);
            }
        }
    }

    // ---- feeding waves.  Panel p holds columns p * PANEL .. of E.  Thread -> (row r, column k of the
    // panel), chosen so that consecutive threads read consecutive memory: rows of E are contiguous
    // unless E is a transpose of the stored block, in which case its columns are.  Element u of a
    // thread's share of panel p is  E(r0 + u ru, c0 + p PANEL + u cu)  at  tbase + p pstep + u ustep:
    // the index maps (transposition, reversal of an upper E) are folded into signed strides once, so
    // that a fetch spends a handful of instructions per element.
    const int r0 = a.etrans ? tid / PANEL : tid % WIDE, ru = a.etrans ? FT / PANEL : 0;
    const int c0 = a.etrans ? tid % PANEL : tid / WIDE, cu = a.etrans ? 0 : FT / WIDE;
    const int64_t sr = (a.etrans ? a.lda : 1) * (e_lower ? 1 : -1), sc = (a.etrans ? 1 : a.lda) * (e_lower ? 1 : -1);
    const T *const tbase = a.A + (e_lower ? 0 : (int64_t)(dim - 1) * (a.lda + 1)) + r0 * sr + c0 * sc;
    const int64_t pstep = PANEL * sc, ustep = ru * sr + cu * sc;
    T stage[DEPTH][EL];
    auto fetch = [&](int p, int slot) {
        const T *ptr = tbase + p * pstep;
        int r = r0, c = c0 + p * PANEL;
#pragma unroll
        for (int u = 0; u < EL; ++u) {
            const int inside = (int)(r < dim) & (int)(r > c);                // strictly lower part of E
            stage[slot][u] = *(inside ? ptr : a.A);                          // looked at in stash, not here: no load is waited for
            ptr += ustep;
            r += ru;
            c += cu;
        }
    };
    // all reads of d_inv come before the first write of the panel: LDS reads and writes keep their order,
    // so a read between two writes would cost a round trip each
    auto stash = [&](int p, int slot) {
        T scale[EL];
        int c = c0 + p * PANEL;
#pragma unroll
        for (int u = 0; u < EL; ++u) {
            scale[u] = d_inv[c < WIDE ? c : 0];                              // column c scaled by 1 / E(c, c)
            c += cu;
        }
        int at = (p & 1) * (PANEL * WIDE) + c0 * WIDE + r0, r = r0;
        c = c0 + p * PANEL;
#pragma unroll
        for (int u = 0; u < EL; ++u) {
            const int inside = (int)(r < dim) & (int)(r > c);
            e_pan[at] = inside ? stage[slot][u] * scale[u] : T(0);
            at += cu * WIDE + ru;
            r += ru;
            c += cu;
        }
    };
    if (feeding) {
#pragma unroll
        for (int sl = 0; sl < DEPTH; ++sl) fetch(sl, sl);
        // diagonal: thread t takes entry t of the stored diagonal
        if (tid < WIDE) {
            const bool has_diag = tid < dim && !a.unit;
            const T dv = a.A[has_diag ? tid + (int64_t)tid * a.lda : 0];
            d_inv[tid < dim ? (e_lower ? tid : dim - 1 - tid) : tid] = has_diag ? T(1) / dv : T(1);
        }
    }
    __syncthreads();                 // d_inv complete
    if (feeding) {
        stash(0, 0);
        fetch(DEPTH, 0);
    }
    __syncthreads();

    // columns of group gc (compile-time), panel by panel; SOLVE and FEED_TOO say which of the two jobs
    // this instance of the code does (both for FEED == 0; otherwise the two kinds of waves run through
    // separate instances, so that neither carries the other's registers, and meet at the barriers)
    auto group = [&](auto gc_tag, auto solve_tag, auto feed_tag) {
        constexpr int gc = decltype(gc_tag)::value;
        constexpr bool SOLVE = decltype(solve_tag)::value, FEED_TOO = decltype(feed_tag)::value;
        constexpr int PER = 64 / PANEL;
#pragma unroll
        for (int pp = 0; pp < PER; ++pp) {
            const int p = gc * PER + pp;
            if (p >= npan) break;    // uniform over the workgroup
            if (SOLVE && live) {
                const T *const pan = e_pan + (p & 1) * (PANEL * WIDE);
                // the multipliers of column k + 1 are read while column k is applied
                T e[GROUPS], e_next[GROUPS];
#pragma unroll
                for (int g = gc; g < GROUPS; ++g) e[g] = pan[lane + 64 * g];
#pragma unroll 2
                for (int k = 0; k < PANEL; ++k) {
                    const int lc = (p * PANEL + k) & 63;                  // lane that holds the pivots
                    const int kn = k + 1 < PANEL ? k + 1 : k;
#pragma unroll
                    for (int g = gc; g < GROUPS; ++g) e_next[g] = pan[kn * WIDE + lane + 64 * g];
#pragma unroll
                    for (int j = 0; j < RPW; ++j) {
                        const T piv = lane_value(y[gc][j], lc);
#pragma unroll
                        for (int g = gc; g < GROUPS; ++g) y[g][j] -= e[g] * piv;
                    }
#pragma unroll
                    for (int g = gc; g < GROUPS; ++g) e[g] = e_next[g];
                }
            }
            if (FEED_TOO && p + 1 < npan) {
                const int slot = (gc * PER + pp + 1) % DEPTH;            // a constant once the loop is unrolled
                stash(p + 1, slot);              // into the half that the solving waves left at the last barrier
                // unconditional (past the last panel it re-reads the block's first element): a fetch that might
                // not have been issued would turn every wait for an older one into a wait for all loads
                fetch(p + 1 + DEPTH, slot);
            }
            __syncthreads();
        }
    };
    auto groups = [&](auto solve_tag, auto feed_tag) {
        group(std::integral_constant<int, 0>{}, solve_tag, feed_tag);
        group(std::integral_constant<int, 1>{}, solve_tag, feed_tag);
        group(std::integral_constant<int, 2>{}, solve_tag, feed_tag);
        group(std::integral_constant<int, 3>{}, solve_tag, feed_tag);
    };
    if (FEED == 0) {
        groups(std::true_type{}, std::true_type{});
    } else if (feeding) {
        groups(std::false_type{}, std::true_type{});
        return;
    } else {
        groups(std::true_type{}, std::false_type{});
    }

    if (!live) return;
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        const int idx = lane + 64 * g;
        if (idx < dim) {
            const T d = d_inv[idx];
#pragma unroll
            for (int j = 0; j < RPW; ++j)
                if (q0 + j < a.nrhs) a.B[xoff[g] + (int64_t)(q0 + j) * qs] = y[g][j] * d;
        }
    }
}

// Diagonal-block product x := alpha E x on the matrix instruction.  E, with zeros
// outside its triangle (ones on an implicit diagonal), sits in LDS and supplies the
// row operands; a wave takes MMA_RHS = 16 right-hand sides, loads them whole as the
// column operands (so that the product may overwrite them) and accumulates the four
// 16-row tiles of the result.  No index reversal is needed here: an upper E is
// simply a matrix with zeros below the diagonal.
constexpr int MMA_RHS = 16;

template <typename T> __global__ void __launch_bounds__(64 * WAVES) trmm_block_kernel(const BlockArgs<T> a) {
    using M = Mma16<T>;
    using acc_t = typename M::acc_t;
    __shared__ T e_cols[NB * NB];            // E(r, c) at [c * NB + r]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lc = lane & 15, lk = lane >> 4;
    const int nbk = a.nbk;
    const int lowr = a.stored_lower ? 1 : 0, unit = a.unit ? 1 : 0;
    constexpr int PER = NB / WAVES;

    // column operands: step s supplies element (4 s + lk) of right-hand side q
    const int q = (blockIdx.x * WAVES + wave) * MMA_RHS + lc;
    const int64_t qs = a.left ? a.ldb : 1, xs = a.left ? 1 : a.ldb;
    T xb[NB / 4];
#pragma unroll
    for (int sx = 0; sx < NB / 4; ++sx) {
        const int row = 4 * sx + lk;
        const bool in = q < a.nrhs && row < nbk;
        const T v = a.B[in ? (int64_t)row * xs + (int64_t)q * qs : 0];
        xb[sx] = in ? v : T(0);
    }
    // thread (wave w, lane t): stored row t, stored columns s = w, w + 4, ...
    T row[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int s = wave + u * WAVES;
        // the referenced triangle, with the diagonal unless it is implicit
        const int tri = (lowr & (int)(lane > s)) | ((lowr ^ 1) & (int)(lane < s)) | ((unit ^ 1) & (int)(lane == s));
        const int inside = (int)(lane < nbk) & (int)(s < nbk) & tri;
        const T v = a.A[(inside ? lane : 0) + (int64_t)(inside ? s : 0) * a.lda];
        row[u] = inside ? v : ((unit & (int)(lane == s) & (int)(lane < nbk)) ? T(1) : T(0));
    }
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int s = wave + u * WAVES;
        const int r = a.etrans ? s : lane, c = a.etrans ? lane : s;
        e_cols[c * NB + r] = row[u];
    }
    __syncthreads();
    if ((blockIdx.x * WAVES + wave) * MMA_RHS >= a.nrhs) return;

    acc_t acc[NB / 16];
#pragma unroll
    for (int t = 0; t < NB / 16; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[t][r] = T(0);
#pragma unroll
    for (int sx = 0; sx < NB / 4; ++sx) {
        if (4 * sx < nbk) {                              // workgroup-uniform: columns of E past the order are zero
#pragma unroll
            for (int t = 0; t < NB / 16; ++t) acc[t] = M::mma(e_cols[(4 * sx + lk) * NB + 16 * t + lc], xb[sx], acc[t]);
        }
    }
    if (q < a.nrhs) {
#pragma unroll
        for (int t = 0; t < NB / 16; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int rr = 16 * t + M::drow(lane, r);
                if (rr < nbk) a.B[(int64_t)rr * xs + (int64_t)q * qs] = a.alpha * acc[t][r];
            }
    }
}

// The same products for diagonal blocks of order up to WIDE = 256.  The workgroup has
// eight multiplying waves and as many feeding waves.  A pair of multiplying waves owns
// MMA_RHS right-hand sides: the upper and the lower eight 16-row tiles of their result
// stay in the accumulators of the one and the other, and the elements of the
// right-hand sides arrive from memory four steps (one panel) at a time, one panel
// ahead of their use; nothing of the result is stored before the last panel, so the
// product may overwrite its input.  E streams through LDS in panels of PANEL columns,
// two halves in turn as in the solve above, written by the feeding waves.
// MODE 0: triangular E with zeros above the diagonal; 1: zeros below; 2: symmetric
// (either triangle stored).  Tiles of E that hold only zeros are passed over.
// One kernel of this kind replaces the four order-64 products and the three coupling
// products between them.
template <typename T> struct WideProdArgs {
    const T *A;      // top-left element of the diagonal block in the stored matrix
    int64_t lda;
    const T *X;      // the block's rows (side L) or columns (side R) of the right-hand sides
    int64_t ldx;
    T *Y;            // where the result goes: the same memory as X (triangular) or the block's part of C (symmetric)
    int64_t ldy;
    int dim, nrhs, left;
    int etrans, stored_lower, unit;   // triangular: E(r,c) = A[c + r*lda] if etrans; symmetric: only stored_lower is read
    T alpha;
    // > 0: the launch covers every diagonal block of order WIDE of a matrix of this order (the last one
    // may be smaller), workgroups (x, y) taking block y; A, X and Y then point at the first block and
    // dim is not read.  Blocks that do not depend on each other only (the symmetric product).
    int batch_order;
};
template <typename T> constexpr size_t wide_prod_lds_bytes() { return 2 * PANEL * WIDE * sizeof(T); }

template <typename T, int MODE>
__global__ void __launch_bounds__(16 * 64) wide_product_kernel(const WideProdArgs<T> a0) {
    WideProdArgs<T> a = a0;
    if (a0.batch_order > 0) {
        const int64_t off = (int64_t)blockIdx.y * WIDE;
        a.A += off + off * a0.lda;
        a.X += a0.left ? off : off * a0.ldx;
        a.Y += a0.left ? off : off * a0.ldy;
        a.dim = (int)(a0.batch_order - off < WIDE ? a0.batch_order - off : WIDE);
    }
    using M = Mma16<T>;
    using acc_t = typename M::acc_t;
    constexpr int DEPTH = 2, TILES = WIDE / 16, HT = TILES / 2, KS = PANEL / 4, NPAN = WIDE / PANEL;
    constexpr int MW = 2 * WAVES, FT = 64 * MW;          // multiplying waves; feeding threads (as many waves again)
    constexpr int EL = PANEL * WIDE / FT;                // elements of a panel per feeding thread
    static_assert(FT == 2 * WIDE && EL * FT == PANEL * WIDE, "two columns of a panel per pass");
    extern __shared__ __align__(16) unsigned char prod_lds[];
    T *const e_pan = reinterpret_cast<T *>(prod_lds);    // E(r, c0 + k) of panel p at [(p & 1) * PANEL * WIDE + k * WIDE + r]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lc = lane & 15, lk = lane >> 4;
    const bool feeding = wave >= MW;                     // wave-uniform
    const int tid = (int)threadIdx.x - (feeding ? FT : 0);   // index within the waves of one kind
    const int dim = a.dim, npan = (dim + PANEL - 1) / PANEL;

    // ---- multiplying waves: wave w takes right-hand sides 16 (w & 3) .. + 15 of the workgroup's 64 and the
    // upper (w < 4) or lower eight 16-row tiles of their result.  Column operands: step sx supplies element
    // (4 sx + lk) of right-hand side q; positions are clamped into the block for the load and sorted out at
    // the point of use.
    const int half = (wave >> 2) & 1, group = wave & (WAVES - 1);
    const int q = (blockIdx.x * WAVES + group) * MMA_RHS + lc;
    const bool live = !feeding && (blockIdx.x * WAVES + group) * MMA_RHS < a.nrhs;
    const int64_t xq = a.left ? a.ldx : 1, xs = a.left ? 1 : a.ldx;
    const T *const xcol = a.X + (int64_t)min(q, a.nrhs - 1) * xq;
    T xr[3][KS];                                         // panel p in xr[p % 3]: asked for two panels before its use
    auto xfetch = [&](int p, int slot) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) xr[slot][ks] = xcol[(int64_t)min(p * PANEL + 4 * ks + lk, dim - 1) * xs];
    };

    // ---- feeding waves: thread -> (row r, column k of the panel) so that consecutive threads read
    // consecutive memory: a thread keeps one row of E and walks every other column of the panel, unless
    // E is the transpose of the stored block, in which case it keeps one column and walks rows.  A fetch
    // reads the stored element behind every position of the panel, also where E holds a zero or an
    // implicit one (positions are clamped into the block, which is memory of the caller's matrix either
    // way); what a position really holds is sorted out when the panel is stored, so that no lane mask has
    // to live from the one to the other.  Only the panel's own 16 rows, the columns past the order and an
    // implicit diagonal need sorting out: rows above them belong to tiles that are never multiplied,
    // rows below are plain entries, and rows past the order only reach results that are not stored.
    const bool by_col = MODE != 2 && a.etrans;
    const int r0 = by_col ? tid / PANEL : tid % WIDE, ru = by_col ? FT / PANEL : 0;
    const int k0 = by_col ? tid % PANEL : tid / WIDE, ku = by_col ? 0 : FT / WIDE;
    int c_next = k0;                                     // column of element 0 of the next panel to fetch
    const int rc = min(r0, dim - 1);                     // the thread's row, clamped (by_col: its first row)
    T stage[DEPTH][EL];
    auto fetch = [&](int slot) {
        if (MODE == 2) {
#pragma unroll
            for (int u = 0; u < EL; ++u) {
                const int c = min(c_next + u * ku, dim - 1);
                const int i = a.stored_lower ? max(rc, c) : min(rc, c), j = a.stored_lower ? min(rc, c) : max(rc, c);
                stage[slot][u] = a.A[i + (int64_t)j * a.lda];
            }
        } else if (!by_col) {
            const T *const rowp = a.A + rc;
#pragma unroll
            for (int u = 0; u < EL; ++u) stage[slot][u] = rowp[(int64_t)min(c_next + u * ku, dim - 1) * a.lda];
        } else {
            const T *const colp = a.A + min(c_next, dim - 1);
#pragma unroll
            for (int u = 0; u < EL; ++u) stage[slot][u] = colp[(int64_t)min(r0 + u * ru, dim - 1) * a.lda];
        }
        c_next += PANEL;
    };
    const int nonunit = a.unit ? 0 : 1;
    auto stash = [&](int p, int slot) {
#pragma unroll
        for (int u = 0; u < EL; ++u) {
            const int r = r0 + u * ru, k = k0 + u * ku, c = p * PANEL + k;
            T v = stage[slot][u];
            if (MODE == 2) {
                v = c < dim ? v : T(0);
            } else {
                const int diag = (int)(r == c), in = (int)(c < dim);
                const int keep = in & ((int)(MODE == 0 ? r > c : r < c) | (diag & nonunit));
                v = keep ? v : ((in & diag) ? T(1) : T(0));     // reached with diag set only for an implicit diagonal
            }
            e_pan[(p & 1) * (PANEL * WIDE) + k * WIDE + r] = v;
        }
    };
    acc_t acc[HT];
    if (feeding) {
#pragma unroll
        for (int sl = 0; sl < DEPTH; ++sl) fetch(sl);    // a panel past the order is read at clamped positions and stored as zeros
        stash(0, 0);
        fetch(0);
        __syncthreads();
    } else {
        xfetch(0, 0);
        xfetch(1, 1);
#pragma unroll
        for (int t = 0; t < HT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[t][r] = T(0);
        __syncthreads();
    }

    // the products of panel p for the half H of the tiles (both compile-time): straight-line code, tiles
    // innermost so that consecutive matrix instructions work on different accumulators
    auto multiply = [&](auto p_tag, auto h_tag) {
        constexpr int p = decltype(p_tag)::value, H = decltype(h_tag)::value;
        const T *const pan = e_pan + (p & 1) * (PANEL * WIDE);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int sx = p * KS + ks;
            const T xv = (4 * sx + lk < dim && q < a.nrhs) ? xr[p % 3][ks] : T(0);
#pragma unroll
            for (int tt = 0; tt < HT; ++tt) {
                const int t = H * HT + tt;
                const bool nonzero = MODE == 0 ? sx <= 4 * t + 3 : MODE == 1 ? sx >= 4 * t : true;   // compile-time
                if (nonzero) acc[tt] = M::mma(pan[(4 * ks + lk) * WIDE + 16 * t + lc], xv, acc[tt]);
            }
        }
    };
    // One step per panel and kind of wave; both kinds meet at the same barriers.  The two kinds run
    // through separate code from here on, so that neither carries the other's registers along.
    auto feed_step = [&](auto p_tag) {
        constexpr int p = decltype(p_tag)::value;
        if (p >= npan) return;                           // uniform over the workgroup
        // unconditional, also past the last panel (positions are clamped, such a panel is stored as zeros into the
        // half that nobody reads any more): a fetch that might not have been issued would turn every wait for an
        // older one into a wait for all loads
        constexpr int slot = (p + 1) % DEPTH;
        stash(p + 1, slot);                              // into the half that nobody reads during this step
        fetch(slot);                                     // panel p + 1 + DEPTH
        __syncthreads();
    };
    auto multiply_step = [&](auto p_tag) {
        constexpr int p = decltype(p_tag)::value;
        if (p >= npan) return;                           // uniform over the workgroup
        if (live) {
            xfetch(p + 2, (p + 2) % 3);                  // positions are clamped into the block: past the last panel it re-reads the last row
            // Every tile of the wave's half takes part whatever the order, in straight-line code.  An
            // earlier form jumped around the tiles past the order, each jump straight after a tile's matrix
            // instruction and all to one block that copies accumulator registers; on that edge the compiler
            // left fewer wait states before the copy than the instruction needs to finish its last-written
            // register pair (it finds the nearest matrix instruction along one path per block only), and
            // rows 12-15 of the last tile missed their final update in some waves.  Rule: no runtime branch
            // between a matrix instruction and the next reader of its accumulator.
            if (half == 0) multiply(p_tag, std::integral_constant<int, 0>{});
            else multiply(p_tag, std::integral_constant<int, 1>{});
        }
        __syncthreads();
    };
    static_assert(NPAN == 16, "sixteen panels, spelled out so that every register index is a constant");
    auto all_panels = [&](auto step) {
        step(std::integral_constant<int, 0>{});
        step(std::integral_constant<int, 1>{});
        step(std::integral_constant<int, 2>{});
        step(std::integral_constant<int, 3>{});
        step(std::integral_constant<int, 4>{});
        step(std::integral_constant<int, 5>{});
        step(std::integral_constant<int, 6>{});
        step(std::integral_constant<int, 7>{});
        step(std::integral_constant<int, 8>{});
        step(std::integral_constant<int, 9>{});
        step(std::integral_constant<int, 10>{});
        step(std::integral_constant<int, 11>{});
        step(std::integral_constant<int, 12>{});
        step(std::integral_constant<int, 13>{});
        step(std::integral_constant<int, 14>{});
        step(std::integral_constant<int, 15>{});
    };
    if (feeding) {
        all_panels(feed_step);
        return;
    }
    all_panels(multiply_step);
    if (q >= a.nrhs) return;
    const int64_t yq = a.left ? a.ldy : 1, ys = a.left ? 1 : a.ldy;
#pragma unroll
    for (int tt = 0; tt < HT; ++tt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int rr = 16 * (half * HT + tt) + M::drow(lane, r);
            if (rr < dim) {
                T *y = a.Y + (int64_t)rr * ys + (int64_t)q * yq;
                *y = MODE == 2 ? *y + a.alpha * acc[tt][r] : a.alpha * acc[tt][r];
            }
        }
}

template <typename T, int MODE> int launch_wide_product(const WideProdArgs<T> &a, void *stream) {
    constexpr size_t LDS = wide_prod_lds_bytes<T>();
    constexpr int PER_WG = MMA_RHS * WAVES;
    const hipError_t e = allow_lds(wide_product_kernel<T, MODE>, LDS);
    if (e != hipSuccess) return (int)e;
    const unsigned blocks = a.batch_order > 0 ? (unsigned)((a.batch_order + WIDE - 1) / WIDE) : 1u;
    hipLaunchKernelGGL((wide_product_kernel<T, MODE>), dim3((unsigned)((a.nrhs + PER_WG - 1) / PER_WG), blocks), dim3(16 * 64),
                       LDS, static_cast<hipStream_t>(stream), a);
    return (int)hipGetLastError();
}

// B := alpha * B (alpha == 0 stores zeros without reading)
template <typename T> __global__ void __launch_bounds__(256) scale_b_kernel(T *B, int64_t ldb, int m, int n, T alpha) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= m) return;
    for (int j = blockIdx.y; j < n; j += gridDim.y) {
        T *p = B + i + (int64_t)j * ldb;
        *p = (alpha == T(0)) ? T(0) : alpha * *p;
    }
}

template <typename T> int real_gemm(char ta, char tb, int64_t m, int64_t n, int64_t k, T alpha, const T *A, int64_t lda,
                                    const T *B, int64_t ldb, T beta, T *C, int64_t ldc, void *stream);
template <> int real_gemm<double>(char ta, char tb, int64_t m, int64_t n, int64_t k, double alpha, const double *A,
                                  int64_t lda, const double *B, int64_t ldb, double beta, double *C, int64_t ldc,
                                  void *stream) {
    return xgemm_dgemm(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream);
}
template <> int real_gemm<float>(char ta, char tb, int64_t m, int64_t n, int64_t k, float alpha, const float *A,
                                 int64_t lda, const float *B, int64_t ldb, float beta, float *C, int64_t ldc,
                                 void *stream) {
    return xgemm_sgemm(ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, stream);
}

template <typename T> struct Tri {
    bool left, stored_lower, trans, unit;
    const T *A;
    int64_t lda;
    T *B;
    int64_t ldb, m, n;
    void *stream;
    bool product;   // false: solve; true: B := alpha op(T) B
    T alpha;        // product only

    // E = op(T) for side L, op(T)^T for side R
    bool etrans() const { return trans != !left; }
    bool e_lower() const { return stored_lower != etrans(); }

    int block(int64_t off, int64_t dim) const {
        BlockArgs<T> a;
        a.A = A + off + off * lda;
        a.lda = lda;
        a.B = left ? B + off : B + off * ldb;
        a.ldb = ldb;
        a.nbk = (int)dim;
        a.nrhs = (int)(left ? n : m);
        a.left = left ? 1 : 0;
        a.etrans = etrans() ? 1 : 0;
        a.stored_lower = stored_lower ? 1 : 0;
        a.unit = unit ? 1 : 0;
        a.alpha = alpha;
        hipStream_t st = static_cast<hipStream_t>(stream);
        const dim3 blk(64 * WAVES);
        auto grid = [&](int rpw) { return dim3((unsigned)((a.nrhs + rpw * WAVES - 1) / (rpw * WAVES))); };
        if (product && dim > NB) {
            WideProdArgs<T> w;
            w.A = a.A;
            w.lda = lda;
            w.X = a.B;
            w.ldx = ldb;
            w.Y = a.B;
            w.ldy = ldb;
            w.dim = a.nbk;
            w.nrhs = a.nrhs;
            w.left = a.left;
            w.etrans = a.etrans;
            w.stored_lower = a.stored_lower;
            w.unit = a.unit;
            w.alpha = alpha;
            w.batch_order = 0;
            return e_lower() ? launch_wide_product<T, 0>(w, stream) : launch_wide_product<T, 1>(w, stream);
        } else if (product) {
            hipLaunchKernelGGL(trmm_block_kernel<T>, grid(MMA_RHS), blk, 0, st, a);
        } else {
            // Right-hand sides per wave: a solve is a chain of dependent steps whose length in time
            // grows with the right-hand sides a wave carries, so few right-hand sides are spread
            // thinly over many waves, and only a count that fills the device is packed densely.
            // (Measured: in double precision 2 per wave win up to about 2048 waves; in single
            // precision, where a pivot costs one lane read instead of two, 4 per wave win throughout.)
            constexpr bool DBL = sizeof(T) == 8;
            constexpr int64_t SOLVE_WAVES = DBL ? 2048 : 4096;
            const int SOLVE_CUS = device_cus();
            auto fits = [&](int rpw) { return (a.nrhs + rpw - 1) / rpw <= SOLVE_WAVES; };
            if (dim <= NB) {
                if (fits(4)) hipLaunchKernelGGL((trsm_block_kernel<T, 4>), grid(4), blk, 0, st, a);
                else if (fits(8)) hipLaunchKernelGGL((trsm_block_kernel<T, 8>), grid(8), blk, 0, st, a);
                else hipLaunchKernelGGL((trsm_block_kernel<T, 16>), grid(16), blk, 0, st, a);
            } else {
                constexpr size_t LDS = wide_lds_bytes<T>();
                hipError_t e = hipSuccess;
                auto go = [&](auto kern, int rpw, int feed, int sw) {
                    if ((e = allow_lds(kern, LDS)) == hipSuccess)
                        hipLaunchKernelGGL(kern, dim3((unsigned)((a.nrhs + rpw * sw - 1) / (rpw * sw))), dim3(64 * (sw + feed)), LDS, st, a);
                };
                // Separate feeding waves pay while a workgroup has a compute unit to itself: four solving
                // and eight feeding waves, with the fewest right-hand sides per wave that still keep the
                // workgroups within the compute units; beyond that, workgroups of four waves that do both.
                // (Eight solving waves with half the right-hand sides each were no faster at 8192
                // right-hand sides and slower at few.)
                auto alone = [&](int rpw) { return (a.nrhs + WAVES * rpw - 1) / (WAVES * rpw) <= SOLVE_CUS; };
                if (DBL && alone(2)) go(trsm_wide_kernel<T, 2, 4, 8, WAVES>, 2, 8, WAVES);
                else if (alone(4)) go(trsm_wide_kernel<T, 4, 3, 8, WAVES>, 4, 8, WAVES);
                else if (alone(8)) go(trsm_wide_kernel<T, 8, 2, 8, WAVES>, 8, 8, WAVES);
                else go(trsm_wide_kernel<T, 8, 2, 0, 4>, 8, 0, 4);
                if (e != hipSuccess) return (int)e;
            }
        }
        return (int)hipGetLastError();
    }

    // part `to` of B += coef * (off-diagonal block of op(T)) applied to part `from`; parts are the
    // rows (side L) or columns (side R) [off, off + n1) = 0 and [off + n1, off + n1 + n2) = 1
    int couple(int64_t off, int64_t n1, int64_t n2, int from, T coef) const {
        // the off-diagonal block of the stored triangle: T21 (n2 x n1) or T12 (n1 x n2)
        const T *blk = stored_lower ? A + (off + n1) + off * lda : A + off + (off + n1) * lda;
        const char tc = trans ? 'T' : 'N';
        const int64_t o[2] = {off, off + n1}, len[2] = {n1, n2};
        const int to = 1 - from;
        if (left)
            return real_gemm<T>(tc, 'N', len[to], n, len[from], coef, blk, lda, B + o[from], ldb, T(1), B + o[to], ldb,
                                stream);
        return real_gemm<T>('N', tc, m, len[to], len[from], coef, B + o[from] * ldb, ldb, blk, lda, T(1),
                            B + o[to] * ldb, ldb, stream);
    }

    // rows/columns [off, off + dim) of the triangular matrix against the matching part of B
    int run(int64_t off, int64_t dim) const {
        if (dim <= WIDE) return block(off, dim);
        const int64_t n1 = ((dim / 2 + NB - 1) / NB) * NB, n2 = dim - n1;
        int rc;
        if (!product) {
            // E lower: x1 = E11^-1 b1;  b2 -= E21 x1;  x2 = E22^-1 b2.   E upper: the other way round.
            const int head = e_lower() ? 0 : 1;
            if ((rc = head == 0 ? run(off, n1) : run(off + n1, n2))) return rc;
            if ((rc = couple(off, n1, n2, head, T(-1)))) return rc;
            return head == 0 ? run(off + n1, n2) : run(off, n1);
        }
        // E lower: b2 := a E22 b2;  b2 += a E21 b1 (b1 still the input);  b1 := a E11 b1.   E upper: the other way round.
        const int head = e_lower() ? 1 : 0;
        if ((rc = head == 0 ? run(off, n1) : run(off + n1, n2))) return rc;
        if ((rc = couple(off, n1, n2, 1 - head, alpha))) return rc;
        return head == 0 ? run(off + n1, n2) : run(off, n1);
    }
};

template <typename T>
int check_tri_args(char side, char uplo, char transa, char diag, int64_t m, int64_t n, T alpha, const T *A, int64_t lda,
                   const T *B, int64_t ldb) {
    const bool left = (side == 'L' || side == 'l'), right = (side == 'R' || side == 'r');
    const bool lower = (uplo == 'L' || uplo == 'l'), upper = (uplo == 'U' || uplo == 'u');
    const bool unit = (diag == 'U' || diag == 'u'), nonunit = (diag == 'N' || diag == 'n');
    if (!left && !right) return -1;
    if (!lower && !upper) return -2;
    if (!is_n(transa) && !is_t(transa)) return -3;
    if (!unit && !nonunit) return -4;
    if (m < 0 || m > DIM_MAX) return -5;
    if (n < 0 || n > DIM_MAX) return -6;
    const bool a_read = alpha != T(0) && m > 0 && n > 0;
    if (a_read && !A) return -8;
    if (lda < max64(1, left ? m : n)) return -9;
    if (m > 0 && n > 0 && !B) return -10;
    if (ldb < max64(1, m)) return -11;
    return 0;
}

template <typename T> int scale_b(T *B, int64_t ldb, int64_t m, int64_t n, T alpha, void *stream) {
    const dim3 grid((unsigned)((m + 255) / 256), (unsigned)(n < 1024 ? n : 1024));
    hipLaunchKernelGGL(scale_b_kernel<T>, grid, dim3(256), 0, static_cast<hipStream_t>(stream), B, ldb, (int)m, (int)n, alpha);
    return (int)hipGetLastError();
}

template <typename T>
int trsm_impl(char side, char uplo, char transa, char diag, int64_t m, int64_t n, T alpha, const T *A, int64_t lda,
              T *B, int64_t ldb, void *stream) {
    const int info = check_tri_args<T>(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb);
    if (info) return info;
    if (m == 0 || n == 0) return 0;
    if (alpha != T(1)) {
        const int rc = scale_b<T>(B, ldb, m, n, alpha, stream);
        if (rc || alpha == T(0)) return rc;
    }
    const bool left = (side == 'L' || side == 'l');
    Tri<T> s{left, uplo == 'L' || uplo == 'l', is_t(transa), diag == 'U' || diag == 'u', A, lda, B, ldb, m, n, stream,
             false, T(1)};
    return s.run(0, left ? m : n);
}

template <typename T>
int trmm_impl(char side, char uplo, char transa, char diag, int64_t m, int64_t n, T alpha, const T *A, int64_t lda,
              T *B, int64_t ldb, void *stream) {
    const int info = check_tri_args<T>(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb);
    if (info) return info;
    if (m == 0 || n == 0) return 0;
    if (alpha == T(0)) return scale_b<T>(B, ldb, m, n, alpha, stream);
    const bool left = (side == 'L' || side == 'l');
    Tri<T> s{left, uplo == 'L' || uplo == 'l', is_t(transa), diag == 'U' || diag == 'u', A, lda, B, ldb, m, n, stream,
             true, alpha};
    return s.run(0, left ? m : n);
}

// ~ 1 / sqrt(d), good to about an ulp for TINY <= d <= BIG, from the hardware's
// estimate y (good to about 2^-23):  h = y / 2 is refined once against g = d y with
// the residual 1/2 - h g (error squared, about 2^-45), then once more against d
// itself with 1/4 - (d h) h.  Seven dependent operations after the estimate, no
// branch, instead of the several dozen of a correctly rounded square root followed
// by a division.  Outside that range (and for zero, negative or non-numeric d) the
// result is not to be used.
template <typename T> static __device__ __forceinline__ T inverse_root(T d) {
    const T y = Mma16<T>::rsq(d);
    const T g = d * y, h = T(0.5) * y;
    const T h1 = __builtin_fma(h, __builtin_fma(-h, g, T(0.5)), h);
    const T e = __builtin_fma(-(d * h1), h1, T(0.25));
    return __builtin_fma(T(4) * h1, e, h1 + h1);
}

// Cholesky factorisation of a diagonal block of order nbk <= NB = 64 by one wave.
//
// The block lives in the registers of the wave as 16x16 tiles in the result layout
// of the matrix instruction (tile rows >= tile columns only), so that the update of
// everything to the right of a finished panel of four columns is one instruction
// per tile,  tile(I, J) -= L(I, panel) L(J, panel)^T,  whose two operands have the
// same register format.  Per panel:
//   1. the four columns leave the tiles through LDS and arrive one row per lane;
//   2. they are factored there: the 4x4 block on the diagonal in every lane alike,
//      from values read out of the lanes that own it, and each lane's own row with
//      the reciprocal pivot roots and the block's entries of L that this yields;
//      no step of it branches.  Pivots outside the range that the reciprocal square
//      root estimate serves, and a ragged last panel, take a column-by-column route
//      with the library's square root and a division instead.  Finished columns go
//      straight to memory;
//   3. the panel returns through LDS in operand format and the tiles are updated.
// After four panels the first tile column is finished and the tiles move up and to
// the left by one, which keeps every register index static while the loops over
// tile columns and panels stay loops (the code stays small: it runs once per
// launch, from a cold instruction cache).  Entries above the diagonal and rows
// above a panel take part with whatever they hold; they only reach entries that
// are finished or never stored.  An upper-stored block (A = U^T U) is the lower
// problem on the transposed block.  A pivot that is not positive stops the block
// and is reported: *info receives base + c + 1 unless an earlier failure is already
// recorded there.
template <typename T>
__global__ void __launch_bounds__(64) potf2_kernel(T *A, int64_t lda, int nbk, int lower, int *info, int base) {
    using M = Mma16<T>;
    using acc_t = typename M::acc_t;
    __builtin_amdgcn_s_setprio(3);                        // see potrf_multi_kernel
    constexpr int TI = NB / 16;                           // tiles per side
    const int lane = threadIdx.x, lc = lane & 15;
    // element (r, c), r >= c, of the lower problem sits at A[r + c*lda] (lower) or A[c + r*lda] (upper)
    const int64_t rs = lower ? 1 : lda, cs = lower ? lda : 1;
    __shared__ T pan[4 * NB];                             // a panel: column k of it at [k * NB + row]

    acc_t acc[TI][TI];
#pragma unroll
    for (int J = 0; J < TI; ++J)
#pragma unroll
        for (int I = J; I < TI; ++I)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 16 * I + M::drow(lane, r), col = 16 * J + lc;
                const bool inside = row < nbk && col <= row;
                const T v = A[inside ? row * rs + col * cs : 0];
                acc[I][J][r] = inside ? v : T(0);
            }

#pragma unroll 1
    for (int J = 0; J < TI; ++J) {
        const int row0 = 16 * J;                          // first row and column of the block that tile (0, 0) holds now
        const int grow = row0 + lane;                     // this lane's row of the block in the one-row-per-lane layout
#pragma unroll 1
        for (int jj = 0; jj < 16; jj += 4) {
            const int c0 = row0 + jj;
            if (c0 >= nbk) return;
            // 1. columns jj .. jj+3 of tile column 0 -> one row per lane
            const int kk = lc - jj;
            if (kk >= 0 && kk < 4) {
#pragma unroll
                for (int I = 0; I < TI; ++I)
#pragma unroll
                    for (int r = 0; r < 4; ++r) pan[kk * NB + 16 * I + M::drow(lane, r)] = acc[I][0][r];
            }
            __builtin_amdgcn_wave_barrier();              // one wave: LDS operations complete in program order
            T pk[4], l[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) pk[k] = pan[k * NB + lane];
            __builtin_amdgcn_wave_barrier();
            // 2. factor the panel.  Fast route, free of branches: the panel's 4x4 diagonal block
            // is read from the lanes that own it and factored in every lane alike (d[k], the
            // pivots; ri[k] ~ 1 / sqrt(d[k]); lik, the block's entries of L), while each lane
            // applies the same operations in the same order to its own row, so that the rows
            // of the diagonal block come out bit for bit as the values used for the others.
            bool fast;
            {
                const T a00 = lane_value(pk[0], jj), a10 = lane_value(pk[0], jj + 1), a20 = lane_value(pk[0], jj + 2),
                        a30 = lane_value(pk[0], jj + 3), a11 = lane_value(pk[1], jj + 1), a21 = lane_value(pk[1], jj + 2),
                        a31 = lane_value(pk[1], jj + 3), a22 = lane_value(pk[2], jj + 2), a32 = lane_value(pk[2], jj + 3),
                        a33 = lane_value(pk[3], jj + 3);
                T d[4], ri[4], q[4];
                d[0] = a00;
                ri[0] = inverse_root<T>(d[0]);
                const T l10 = a10 * ri[0], l20 = a20 * ri[0], l30 = a30 * ri[0];
                d[1] = __builtin_fma(-l10, l10, a11);
                ri[1] = inverse_root<T>(d[1]);
                const T l21 = __builtin_fma(-l20, l10, a21) * ri[1], l31 = __builtin_fma(-l30, l10, a31) * ri[1];
                d[2] = __builtin_fma(-l21, l21, __builtin_fma(-l20, l20, a22));
                ri[2] = inverse_root<T>(d[2]);
                const T l32 = __builtin_fma(-l31, l21, __builtin_fma(-l30, l20, a32)) * ri[2];
                d[3] = __builtin_fma(-l32, l32, __builtin_fma(-l31, l31, __builtin_fma(-l30, l30, a33)));
                ri[3] = inverse_root<T>(d[3]);
                q[0] = pk[0] * ri[0];
                q[1] = __builtin_fma(-q[0], l10, pk[1]) * ri[1];
                q[2] = __builtin_fma(-q[1], l21, __builtin_fma(-q[0], l20, pk[2])) * ri[2];
                q[3] = __builtin_fma(-q[2], l32, __builtin_fma(-q[1], l31, __builtin_fma(-q[0], l30, pk[3]))) * ri[3];
                // valid if all four columns exist and every pivot is in the range the estimate serves
                // (a pivot that is zero, negative or not a number fails the first comparison)
                int valid = (int)(c0 + 4 <= nbk);
#pragma unroll
                for (int k = 0; k < 4; ++k) valid &= (int)(d[k] >= M::TINY) & (int)(d[k] <= M::BIG);
                fast = valid != 0;
                if (fast) {                               // wave-uniform
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const T g = d[k] * ri[k];         // the diagonal entry: one correction step on d ri
                        const T s = __builtin_fma(__builtin_fma(-g, g, d[k]), T(0.5) * ri[k], g);
                        l[k] = q[k];
                        if (lane >= jj + k && grow < nbk) A[grow * rs + (c0 + k) * cs] = lane == jj + k ? s : q[k];
                    }
                }
            }
            // Careful route, column by column: the block's last panel when the order is not a
            // multiple of four, pivots that are tiny, huge or not positive.
            if (!fast) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int piv = jj + k;               // lane that holds the pivot row
                    l[k] = T(0);
                    if (c0 + k < nbk) {                   // wave-uniform
                        const T d = lane_value(pk[k], piv);
                        if (!(d > T(0))) {
                            if (lane == 0 && *info == 0) *info = base + c0 + k + 1;
                            return;
                        }
                        const T s = sqrt(d);
                        l[k] = lane == piv ? s : pk[k] / s;
                        if (lane >= piv && grow < nbk) A[grow * rs + (c0 + k) * cs] = l[k];
#pragma unroll
                        for (int k2 = k + 1; k2 < 4; ++k2) pk[k2] -= l[k] * lane_value(l[k], jj + k2);
                    }
                }
            }
            // 3. the panel in operand format: lane t gets L(16 I + (t & 15), c0 + (t >> 4))
#pragma unroll
            for (int k = 0; k < 4; ++k) pan[k * NB + lane] = l[k];
            __builtin_amdgcn_wave_barrier();
            T op[TI], nop[TI];
#pragma unroll
            for (int I = 0; I < TI; ++I) {
                op[I] = pan[(lane >> 4) * NB + 16 * I + lc];
                nop[I] = -op[I];
            }
            __builtin_amdgcn_wave_barrier();
            const int live = TI - J;                      // tile rows and columns that still hold part of the block
#pragma unroll
            for (int J2 = 0; J2 < TI; ++J2) {
                if (J2 < live && (J2 > 0 || jj < 12)) {   // wave-uniform; the first tile column is finished after its last panel
#pragma unroll
                    for (int I = J2; I < TI; ++I) acc[I][J2] = M::mma(nop[I], op[J2], acc[I][J2]);
                }
            }
        }
        // the first tile row and column are finished: everything moves up and to the left by one tile
#pragma unroll
        for (int J2 = 0; J2 + 1 < TI; ++J2)
#pragma unroll
            for (int I = J2; I + 1 < TI; ++I) acc[I][J2] = acc[I + 1][J2 + 1];
#pragma unroll
        for (int J2 = 0; J2 < TI; ++J2)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[TI - 1][J2][r] = T(0);
    }
}

// Cholesky factorisation of a diagonal block of order nbk <= 64 NBLK by one workgroup of
// NBLK (NBLK + 1) / 2 waves: one wave per 64x64 block of the lower triangle, which holds
// its block in 16x16 accumulator tiles from start to end (the diagonal blocks as in
// potf2_kernel, tile rows >= tile columns only).  Block column jc is worked through in
// panels of four columns; per panel
//   A  the wave of the diagonal block (jc, jc) factors the panel exactly as potf2_kernel
//      does, and leaves in LDS the finished panel in operand format and the scalars that
//      the rows below need (reciprocal pivot roots and the 4x4 block's entries of L; pivot
//      roots instead on the careful route);
//   B  each wave (bi, jc) below it takes its 64 rows of the panel out of its tiles, applies
//      those scalars (one row per lane, the same operations as the diagonal wave applies
//      to its own rows), stores them, leaves them in LDS in operand format and updates
//      the rest of its block;
//   C  each wave (bi, bj), bj > jc, subtracts L(bi, panel) L(bj, panel)^T from its block:
//      one instruction per tile, operands read from LDS.
// The three run as a pipeline, A on panel s while B is on s - 1 and C on s - 2, with one
// workgroup barrier per step and the LDS panels in a ring of three, so a block column costs
// 18 steps of about the time potf2_kernel takes per panel whatever NBLK is.  When a block
// column is done the diagonal block of the next one has received all its updates and
// its wave turns from C to A.  Waves whose blocks lie beyond nbk, or whose block column is
// finished, only keep the barriers company.  A pivot that is not positive is reported as in
// potf2_kernel and ends all further work (never the barriers).
template <typename T, int NBLK>
__global__ void __launch_bounds__(64 * NBLK * (NBLK + 1) / 2)
potrf_multi_kernel(T *A, int64_t lda, int nbk, int lower, int *info, int base) {
    using M = Mma16<T>;
    using acc_t = typename M::acc_t;
    // a chain of dependent steps that the factorisation of a whole matrix waits for: where its waves share
    // a SIMD with those of a concurrent update, they go first
    __builtin_amdgcn_s_setprio(3);
    constexpr int RING = 3, PANELS = 16, STEPS = PANELS + 2, BS = 64;
    const int lane = threadIdx.x & 63, lc = lane & 15, lk = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    int bi = 0;
    while ((bi + 1) * (bi + 2) / 2 <= wave) ++bi;
    const int bj = wave - bi * (bi + 1) / 2;
    const int64_t rs = lower ? 1 : lda, cs = lower ? lda : 1;
    __shared__ T panL[NBLK][RING][4 * BS];   // finished panels of each block row, column k at [k * BS + row]
    __shared__ T panX[NBLK][4 * BS];         // a block row's way from tiles to one row per lane
    __shared__ T scal[RING][16];             // [0] route (0 none, 1 fast, 2 careful), [1] columns, [2..5] roots, [6..11] block entries
    __shared__ int dead;
    if (threadIdx.x == 0) dead = 0;
    __syncthreads();

    auto run = [&](auto diag_tag) {
        constexpr bool DIAG = decltype(diag_tag)::value;
        acc_t acc[4][4];
#pragma unroll
        for (int J = 0; J < 4; ++J)
#pragma unroll
            for (int I = DIAG ? J : 0; I < 4; ++I)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = BS * bi + 16 * I + M::drow(lane, r), col = BS * bj + 16 * J + lc;
                    const bool inside = row < nbk && col <= row;
                    const T v = A[inside ? row * rs + col * cs : 0];
                    acc[I][J][r] = inside ? v : T(0);
                }

        // C: block (bi, bj) -= L(bi, panel) L(bj, panel)^T
        auto trailing = [&](int slot) {
            const T *rowp = &panL[bi][slot][lk * BS + lc], *colp = &panL[bj][slot][lk * BS + lc];
            T op[4], nop[4];
#pragma unroll
            for (int I = 0; I < 4; ++I) {
                nop[I] = -rowp[16 * I];
                op[I] = colp[16 * I];
            }
#pragma unroll
            for (int J = 0; J < 4; ++J)
#pragma unroll
                for (int I = DIAG ? J : 0; I < 4; ++I) acc[I][J] = M::mma(nop[I], op[J], acc[I][J]);
        };

        // A: panel p of the diagonal block (DIAG only); tile (0, 0) holds the rows and columns from 16 (p / 4) on
        auto factor = [&](int jc, int p) {
            const int slot = p % RING, jj = 4 * (p & 3), row0 = BS * jc + 16 * (p >> 2), c0 = row0 + jj;
            const int grow = row0 + lane;
            const int rlim = nbk < BS * (jc + 1) ? nbk : BS * (jc + 1);   // rows of this block
            T *const px = &panX[bi][0], *const pl = &panL[bi][slot][0];
            const int kk = lc - jj;
            if (kk >= 0 && kk < 4) {
#pragma unroll
                for (int I = 0; I < 4; ++I)
#pragma unroll
                    for (int r = 0; r < 4; ++r) px[kk * BS + 16 * I + M::drow(lane, r)] = acc[I][0][r];
            }
            __builtin_amdgcn_wave_barrier();
            T pk[4], l[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) pk[k] = px[k * BS + lane];
            __builtin_amdgcn_wave_barrier();
            bool fast;
            {
                const T a00 = lane_value(pk[0], jj), a10 = lane_value(pk[0], jj + 1), a20 = lane_value(pk[0], jj + 2),
                        a30 = lane_value(pk[0], jj + 3), a11 = lane_value(pk[1], jj + 1), a21 = lane_value(pk[1], jj + 2),
                        a31 = lane_value(pk[1], jj + 3), a22 = lane_value(pk[2], jj + 2), a32 = lane_value(pk[2], jj + 3),
                        a33 = lane_value(pk[3], jj + 3);
                T d[4], ri[4], q[4];
                d[0] = a00;
                ri[0] = inverse_root<T>(d[0]);
                const T l10 = a10 * ri[0], l20 = a20 * ri[0], l30 = a30 * ri[0];
                d[1] = __builtin_fma(-l10, l10, a11);
                ri[1] = inverse_root<T>(d[1]);
                const T l21 = __builtin_fma(-l20, l10, a21) * ri[1], l31 = __builtin_fma(-l30, l10, a31) * ri[1];
                d[2] = __builtin_fma(-l21, l21, __builtin_fma(-l20, l20, a22));
                ri[2] = inverse_root<T>(d[2]);
                const T l32 = __builtin_fma(-l31, l21, __builtin_fma(-l30, l20, a32)) * ri[2];
                d[3] = __builtin_fma(-l32, l32, __builtin_fma(-l31, l31, __builtin_fma(-l30, l30, a33)));
                ri[3] = inverse_root<T>(d[3]);
                q[0] = pk[0] * ri[0];
                q[1] = __builtin_fma(-q[0], l10, pk[1]) * ri[1];
                q[2] = __builtin_fma(-q[1], l21, __builtin_fma(-q[0], l20, pk[2])) * ri[2];
                q[3] = __builtin_fma(-q[2], l32, __builtin_fma(-q[1], l31, __builtin_fma(-q[0], l30, pk[3]))) * ri[3];
                int valid = (int)(c0 + 4 <= nbk);
#pragma unroll
                for (int k = 0; k < 4; ++k) valid &= (int)(d[k] >= M::TINY) & (int)(d[k] <= M::BIG);
                fast = valid != 0;
                if (fast) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const T g = d[k] * ri[k];
                        const T sd = __builtin_fma(__builtin_fma(-g, g, d[k]), T(0.5) * ri[k], g);
                        l[k] = q[k];
                        if (lane >= jj + k && grow < rlim) A[grow * rs + (c0 + k) * cs] = lane == jj + k ? sd : q[k];
                    }
                    if (lane == 0) {
                        T *sc = &scal[slot][0];
                        sc[0] = T(1);
                        sc[1] = T(4);
#pragma unroll
                        for (int k = 0; k < 4; ++k) sc[2 + k] = ri[k];
                        sc[6] = l10; sc[7] = l20; sc[8] = l30; sc[9] = l21; sc[10] = l31; sc[11] = l32;
                    }
                }
            }
            if (!fast) {
                int done = 0;
                bool failed = false;
                T sq[4] = {T(1), T(1), T(1), T(1)}, lb[6] = {T(0), T(0), T(0), T(0), T(0), T(0)};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int piv = jj + k;
                    l[k] = T(0);
                    if (!failed && c0 + k < nbk) {            // wave-uniform
                        const T d = lane_value(pk[k], piv);
                        if (!(d > T(0))) {
                            if (lane == 0 && *info == 0) *info = base + c0 + k + 1;
                            failed = true;
                        } else {
                            const T sd = sqrt(d);
                            sq[k] = sd;
                            l[k] = lane == piv ? sd : pk[k] / sd;
                            if (lane >= piv && grow < rlim) A[grow * rs + (c0 + k) * cs] = l[k];
                            int e = k == 0 ? 0 : k == 1 ? 3 : 5;   // entries (k+1.., k) of the block: 6 + {0,1,2}, {3,4}, {5}
#pragma unroll
                            for (int k2 = k + 1; k2 < 4; ++k2) {
                                const T x = lane_value(l[k], jj + k2);
                                lb[e++] = x;
                                pk[k2] -= l[k] * x;
                            }
                            done = k + 1;
                        }
                    }
                }
                if (lane == 0) {
                    T *sc = &scal[slot][0];
                    sc[0] = failed ? T(0) : T(2);
                    sc[1] = (T)done;
#pragma unroll
                    for (int k = 0; k < 4; ++k) sc[2 + k] = sq[k];
#pragma unroll
                    for (int e = 0; e < 6; ++e) sc[6 + e] = lb[e];
                    if (failed) dead = 1;
                }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) pl[k * BS + lane] = l[k];
            __builtin_amdgcn_wave_barrier();
            T op[4], nop[4];
#pragma unroll
            for (int I = 0; I < 4; ++I) {
                op[I] = pl[lk * BS + 16 * I + lc];
                nop[I] = -op[I];
            }
            const int live = 4 - (p >> 2);
#pragma unroll
            for (int J2 = 0; J2 < 4; ++J2) {
                if (J2 < live && (J2 > 0 || jj < 12)) {
#pragma unroll
                    for (int I = J2; I < 4; ++I) acc[I][J2] = M::mma(nop[I], op[J2], acc[I][J2]);
                }
            }
        };
        // after four panels the first tile row and column of a diagonal block are finished: up and to the left by one tile
        auto shift_diag = [&]() {
#pragma unroll
            for (int J2 = 0; J2 + 1 < 4; ++J2)
#pragma unroll
                for (int I = J2; I + 1 < 4; ++I) acc[I][J2] = acc[I + 1][J2 + 1];
#pragma unroll
            for (int J2 = 0; J2 < 4; ++J2)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[3][J2][r] = T(0);
        };

        // B: panel p of block (bi, jc) below the diagonal block (not DIAG); tile column 0 holds the columns from 16 (p / 4) on
        auto below = [&](int jc, int p) {
            const int slot = p % RING, jj = 4 * (p & 3), c0 = BS * jc + 16 * (p >> 2) + jj;
            const int grow = BS * bi + lane;
            T *const px = &panX[bi][0], *const pl = &panL[bi][slot][0];
            const T *sc = &scal[slot][0];
            const int route = (int)lane_value(sc[0], 0), cols = (int)lane_value(sc[1], 0);
            if (route == 0) return;
            const int kk = lc - jj;
            if (kk >= 0 && kk < 4) {
#pragma unroll
                for (int I = 0; I < 4; ++I)
#pragma unroll
                    for (int r = 0; r < 4; ++r) px[kk * BS + 16 * I + M::drow(lane, r)] = acc[I][0][r];
            }
            __builtin_amdgcn_wave_barrier();
            T pk[4], l[4], root[4], lb[6];
#pragma unroll
            for (int k = 0; k < 4; ++k) pk[k] = px[k * BS + lane];
#pragma unroll
            for (int k = 0; k < 4; ++k) root[k] = lane_value(sc[2 + k], 0);
#pragma unroll
            for (int e = 0; e < 6; ++e) lb[e] = lane_value(sc[6 + e], 0);
            __builtin_amdgcn_wave_barrier();
            if (route == 1) {
                l[0] = pk[0] * root[0];
                l[1] = __builtin_fma(-l[0], lb[0], pk[1]) * root[1];
                l[2] = __builtin_fma(-l[1], lb[3], __builtin_fma(-l[0], lb[1], pk[2])) * root[2];
                l[3] = __builtin_fma(-l[2], lb[5], __builtin_fma(-l[1], lb[4], __builtin_fma(-l[0], lb[2], pk[3]))) * root[3];
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    l[k] = T(0);
                    if (k < cols) {                           // wave-uniform
                        l[k] = pk[k] / root[k];
                        int e = k == 0 ? 0 : k == 1 ? 3 : 5;
#pragma unroll
                        for (int k2 = k + 1; k2 < 4; ++k2) pk[k2] -= l[k] * lb[e++];
                    }
                }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (k < cols && grow < nbk) A[grow * rs + (c0 + k) * cs] = l[k];
                pl[k * BS + lane] = l[k];
            }
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_sched_barrier(0);   // the operands below are not to be fetched while the panel's values are still held
            const T *dp = &panL[jc][slot][lk * BS + lc];
            T op[4], nop[4];
#pragma unroll
            for (int I = 0; I < 4; ++I) {
                nop[I] = -pl[lk * BS + 16 * I + lc];
                op[I] = dp[16 * I];
            }
            const int live = 4 - (p >> 2);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (t < live && (t > 0 || jj < 12)) {
#pragma unroll
                    for (int I = 0; I < 4; ++I) acc[I][t] = M::mma(nop[I], op[t], acc[I][t]);
                }
            }
        };
        // after four panels the first tile column of a block below the diagonal is finished: to the left by one tile
        auto shift_below = [&]() {
#pragma unroll
            for (int t = 0; t + 1 < 4; ++t)
#pragma unroll
                for (int I = 0; I < 4; ++I) acc[I][t] = acc[I][t + 1];
#pragma unroll
            for (int I = 0; I < 4; ++I)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[I][3][r] = T(0);
        };

        // Every wave passes NBLK * STEPS barriers.  The roles have loops of their own so that the
        // tile shifts sit at fixed places in straight code (a shift under a condition would keep two
        // copies of the block alive).
        auto alive = [&]() { return dead == 0 && BS * bi < nbk; };   // the same for every lane of the wave
#pragma unroll 1
        for (int jc = 0; jc < bj; ++jc) {                 // C: block columns to the left of this block
#pragma unroll 1
            for (int s = 0; s < STEPS; ++s) {
                const int p = s - 2;
                if (p >= 0 && alive() && BS * jc + 4 * p < nbk) trailing(p % RING);
                __syncthreads();
            }
        }
        if constexpr (DIAG) {                             // A: this block's own column
#pragma unroll 1
            for (int q = 0; q < 4; ++q) {
#pragma unroll 1
                for (int u = 0; u < 4; ++u) {
                    const int p = 4 * q + u;
                    if (alive() && BS * bj + 4 * p < nbk) factor(bj, p);
                    __syncthreads();
                }
                shift_diag();
            }
            __syncthreads();
            __syncthreads();
        } else {                                          // B: one step behind the diagonal wave
            __syncthreads();
#pragma unroll 1
            for (int q = 0; q < 4; ++q) {
#pragma unroll 1
                for (int u = 0; u < 4; ++u) {
                    const int p = 4 * q + u;
                    if (alive() && BS * bj + 4 * p < nbk) below(bj, p);
                    __syncthreads();
                }
                shift_below();
            }
            __syncthreads();
        }
#pragma unroll 1
        for (int n = (NBLK - 1 - bj) * STEPS; n > 0; --n) __syncthreads();   // finished: keep the others' barriers company
    };
    if (bi == bj) run(std::true_type{});
    else run(std::false_type{});
}

__global__ void clear_info_kernel(int *info) { *info = 0; }

thread_local int64_t t_potrf_block = 256;   // largest order handed to one workgroup (64, 128 or 256)

int syrk_call(char uplo, char trans, int64_t n, int64_t k, double alpha, const double *A, int64_t lda, double beta,
              double *C, int64_t ldc, void *stream) {
    return xgemm_dsyrk(uplo, trans, n, k, alpha, A, lda, beta, C, ldc, stream);
}
int syrk_call(char uplo, char trans, int64_t n, int64_t k, float alpha, const float *A, int64_t lda, float beta,
              float *C, int64_t ldc, void *stream) {
    return xgemm_ssyrk(uplo, trans, n, k, alpha, A, lda, beta, C, ldc, stream);
}

// A11 = L11 L11^T;  A21 := A21 L11^-T;  A22 -= A21 A21^T;  then the same on A22
// (upper:  A11 = U11^T U11;  A12 := U11^-T A12;  A22 -= A12^T A12).
template <typename T> int potrf_run(bool lower, int64_t off, int64_t dim, T *A, int64_t lda, int *info, void *stream) {
    T *D = A + off + off * lda;
    if (dim <= NB) {
        hipLaunchKernelGGL(potf2_kernel<T>, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), D, lda, (int)dim,
                           lower ? 1 : 0, info, (int)off);
        return (int)hipGetLastError();
    }
    if (dim <= 2 * NB && dim <= t_potrf_block) {
        hipLaunchKernelGGL((potrf_multi_kernel<T, 2>), dim3(1), dim3(3 * 64), 0, static_cast<hipStream_t>(stream), D, lda,
                           (int)dim, lower ? 1 : 0, info, (int)off);
        return (int)hipGetLastError();
    }
    // ten waves leave each 168 registers, which the fp64 blocks (128 for the tiles alone) do not fit
    if constexpr (sizeof(T) == 4) {
        if (dim <= 4 * NB && dim <= t_potrf_block) {
            hipLaunchKernelGGL((potrf_multi_kernel<T, 4>), dim3(1), dim3(10 * 64), 0, static_cast<hipStream_t>(stream), D,
                               lda, (int)dim, lower ? 1 : 0, info, (int)off);
            return (int)hipGetLastError();
        }
    }
    const int64_t n1 = ((dim / 2 + NB - 1) / NB) * NB, n2 = dim - n1;
    int rc;
    if ((rc = potrf_run<T>(lower, off, n1, A, lda, info, stream))) return rc;
    T *P = lower ? D + n1 : D + n1 * lda;        // A21 (n2 x n1) or A12 (n1 x n2)
    T *D2 = D + n1 + n1 * lda;
    if (lower) {
        if ((rc = trsm_impl<T>('R', 'L', 'T', 'N', n2, n1, T(1), D, lda, P, lda, stream))) return rc;
        if ((rc = syrk_call('L', 'N', n2, n1, T(-1), P, lda, T(1), D2, lda, stream))) return rc;
    } else {
        if ((rc = trsm_impl<T>('L', 'U', 'T', 'N', n1, n2, T(1), D, lda, P, lda, stream))) return rc;
        if ((rc = syrk_call('U', 'T', n2, n1, T(-1), P, lda, T(1), D2, lda, stream))) return rc;
    }
    return potrf_run<T>(lower, off + n1, n2, A, lda, info, stream);
}

// Two more streams of this host thread on the current device, with the events that tie them to
// the caller's stream and to each other.  Created on first use and kept for the life of the
// process.  Waiting on an event means waiting for its latest record at the time of the call, so a
// handful of events used in turn serve any number of steps.
struct SideLanes {
    static constexpr int RING = 4, KINDS = 5;
    hipStream_t stream[2] = {nullptr, nullptr};
    hipEvent_t fork = nullptr, join[2] = {nullptr, nullptr}, ev[KINDS][RING] = {};
    bool ready = false;
};
SideLanes *side_lanes_slot(int dev) {
    constexpr int MAX_DEV = 64;
    thread_local SideLanes lanes[MAX_DEV];
    return (dev < 0 || dev >= MAX_DEV) ? nullptr : &lanes[dev];
}
SideLanes *side_lanes() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || !side_lanes_slot(dev)) return nullptr;
    SideLanes &ln = *side_lanes_slot(dev);
    if (!ln.ready) {
        for (hipStream_t &st : ln.stream)
            if (!st && hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess) return nullptr;
        auto make = [](hipEvent_t &e) { return e || hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess; };
        bool ok = make(ln.fork) && make(ln.join[0]) && make(ln.join[1]);
        for (auto &kind : ln.ev)
            for (hipEvent_t &e : kind) ok = ok && make(e);
        if (!ok) return nullptr;
        ln.ready = true;
    }
    return &ln;
}

// Gives back what side_lanes() created for this thread on the current device.  The streams are idle
// between calls (every call joins them to the caller's stream), but that join may not have run yet.
int release_side_lanes() {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    SideLanes *ln = side_lanes_slot(dev);
    if (!ln) return (int)hipErrorInvalidDevice;
    hipError_t first = hipSuccess;
    auto note = [&](hipError_t x) { if (first == hipSuccess && x != hipSuccess) first = x; };
    for (hipStream_t &st : ln->stream)
        if (st) { note(hipStreamSynchronize(st)); note(hipStreamDestroy(st)); st = nullptr; }
    auto drop = [&](hipEvent_t &ev) { if (ev) { note(hipEventDestroy(ev)); ev = nullptr; } };
    drop(ln->fork);
    drop(ln->join[0]);
    drop(ln->join[1]);
    for (auto &kind : ln->ev)
        for (hipEvent_t &ev : kind) drop(ev);
    ln->ready = false;
    return (int)first;
}

thread_local int64_t t_potrf_panel = -1;   // -1: by the order; 0: the recursion on one stream; W > 0: panels of W columns

// What to do with a block of order n: a panel width W > 0 for the look-ahead sweep, 0 for the plain
// recursion, HALVE to split it in two first.  Narrow panels keep the chain of dependent small
// kernels short, wide ones keep the trailing updates deep enough to run at the product kernel's
// rate, and above some order the recursion's very deep updates win over any sweep; where these
// cross over was measured (fp64: sweep 37.2 ms against 39.5 at 16384, 208.6 against 203.6 at 32768).
constexpr int64_t HALVE = -2;
template <typename T> int64_t potrf_panel(int64_t n) {
    if (t_potrf_panel >= 0) return t_potrf_panel;
    if (n < 3072) return 0;
    if (n <= 16384) return (sizeof(T) == 8 && n >= 12288) ? 512 : 256;   // fp64 16384: 33.8 ms with 256, 32.3 with 512; 12288: 17.0, 16.8
    return sizeof(T) == 8 ? HALVE : 512;
}

// Right-looking factorisation with look-ahead.  Panel p (W columns) goes through
//   F_p   factor the diagonal block                                              chain stream
//   t_p   solve for the block of the next panel's rows (or columns) beside it    chain stream
//   u_p   update the diagonal block of panel p + 1 with it                       chain stream, after B_{p-1}
//   T_p   solve for all blocks further on                                        side stream, after F_p
//   U_p   update the rest of block column (row) p + 1 with panel p               side stream, after t_p and B_{p-1}
//   B_p   update everything beyond block column p + 1                            caller's stream, after T_p
// and t_{p+1} waits for U_p.  The chain F -> t -> u -> F is all that is serial from panel to
// panel; the solves and updates over the full height of the panel run beside it, and the
// bulk of the arithmetic, B_p, beside both.  B_{p-1}, u_p and U_p add into block column p + 1,
// hence their order; all other pairs that may overlap touch different blocks.  The two
// streams of the library branch off the caller's at the start and are joined to it at the end,
// so to the caller (and to a graph capture of its stream) the call behaves like work on that
// stream alone.
template <typename T>
int potrf_ahead(bool lower, int64_t off, int64_t n, int64_t W, T *A, int64_t lda, int *info, hipStream_t s0) {
    // Under stream capture everything goes to the caller's stream and no event is touched: the
    // same kernels in the same order on the data, so a replay gives the eager bits.  (Ending a
    // capture that spanned the library's streams crashed in the runtime.)
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s0, &capturing) != hipSuccess) return (int)hipGetLastError();
    const bool alone = capturing != hipStreamCaptureStatusNone;
    SideLanes *ln = alone ? nullptr : side_lanes();
    if (!alone && !ln) return (int)hipErrorNotReady;
    hipStream_t s1 = alone ? s0 : ln->stream[0], s2 = alone ? s0 : ln->stream[1];
    enum { FACTORED = 0, NEAR_SOLVED = 1, FAR_SOLVED = 2, FAR_UPDATED = 3, BULK_UPDATED = 4 };
    auto record = [&](int kind, int slot, hipStream_t st) { return alone ? hipSuccess : hipEventRecord(ln->ev[kind][slot], st); };
    auto wait_for = [&](hipStream_t st, int kind, int slot) { return alone ? hipSuccess : hipStreamWaitEvent(st, ln->ev[kind][slot], 0); };
    if (!alone) {
        hipError_t e;
        if ((e = hipEventRecord(ln->fork, s0)) != hipSuccess) return (int)e;
        if ((e = hipStreamWaitEvent(s1, ln->fork, 0)) != hipSuccess) return (int)e;
        if ((e = hipStreamWaitEvent(s2, ln->fork, 0)) != hipSuccess) return (int)e;
    }
    int rc = 0;
    auto ok = [&](hipError_t err) { if (rc == 0 && err != hipSuccess) rc = (int)err; return rc == 0; };
    auto solve = [&](int64_t cnt, const T *D, T *P, hipStream_t st) {
        return lower ? trsm_impl<T>('R', 'L', 'T', 'N', cnt, (int64_t)(W), T(1), D, lda, P, lda, st)
                     : trsm_impl<T>('L', 'U', 'T', 'N', (int64_t)(W), cnt, T(1), D, lda, P, lda, st);
    };
    int step = 0;
    for (int64_t j = 0; j < n && rc == 0; j += W, ++step) {
        const int64_t nj = (n - j) < W ? (n - j) : W, rest = n - j - nj;
        const int slot = step % SideLanes::RING, prev = (step + SideLanes::RING - 1) % SideLanes::RING;
        T *D = A + (off + j) + (off + j) * lda;
        if ((rc = potrf_run<T>(lower, off + j, nj, A, lda, info, s1)) || rest == 0) break;
        // rest > 0 means this panel is a full one (nj == W), and so was every panel before it, each with a B
        const int64_t w2 = rest < W ? rest : W, far = rest - w2;
        const int64_t along = lower ? 1 : lda;             // step from one block to the next along the panel
        T *P1 = lower ? D + nj : D + nj * lda;             // blocks of panel p + 1's rows (columns): w2 x nj (nj x w2)
        T *P2 = P1 + w2 * along;                           // the blocks further on: far x nj (nj x far)
        T *D2 = D + nj + nj * lda;                         // diagonal block of panel p + 1
        T *C2 = lower ? D2 + w2 : D2 + w2 * lda;           // rest of its block column (row)
        T *D3 = D2 + w2 + w2 * lda;
        if (!ok(record(FACTORED, slot, s1))) break;
        // the near solve reads what U_{p-1} has updated (the factorisation above did not have to wait for that)
        if (step > 0 && !ok(wait_for(s1, FAR_UPDATED, prev))) break;
        if ((rc = solve(w2, D, P1, s1)) || !ok(record(NEAR_SOLVED, slot, s1))) break;
        if (far > 0) {
            if (!ok(wait_for(s2, FACTORED, slot))) break;
            if ((rc = solve(far, D, P2, s2)) || !ok(record(FAR_SOLVED, slot, s2))) break;
        }
        if (step > 0 && !ok(wait_for(s1, BULK_UPDATED, prev))) break;
        if ((rc = lower ? syrk_call('L', 'N', w2, nj, T(-1), P1, lda, T(1), D2, lda, s1)
                        : syrk_call('U', 'T', w2, nj, T(-1), P1, lda, T(1), D2, lda, s1)))
            break;
        if (far > 0) {
            if (!ok(wait_for(s2, NEAR_SOLVED, slot))) break;
            if (step > 0 && !ok(wait_for(s2, BULK_UPDATED, prev))) break;
            rc = lower ? real_gemm<T>('N', 'T', far, w2, nj, T(-1), P2, lda, P1, lda, T(1), C2, lda, s2)
                       : real_gemm<T>('T', 'N', w2, far, nj, T(-1), P1, lda, P2, lda, T(1), C2, lda, s2);
            if (rc || !ok(record(FAR_UPDATED, slot, s2))) break;
            if (!ok(wait_for(s0, FAR_SOLVED, slot))) break;
            rc = lower ? syrk_call('L', 'N', far, nj, T(-1), P2, lda, T(1), D3, lda, s0)
                       : syrk_call('U', 'T', far, nj, T(-1), P2, lda, T(1), D3, lda, s0);
            if (rc || !ok(record(BULK_UPDATED, slot, s0))) break;
        }
    }
    // both streams always rejoin the caller's, whatever happened above
    hipError_t ej = hipSuccess;
    for (int i = 0; i < 2 && !alone; ++i) {
        hipError_t x = hipEventRecord(ln->join[i], ln->stream[i]);
        if (x == hipSuccess) x = hipStreamWaitEvent(s0, ln->join[i], 0);
        if (ej == hipSuccess) ej = x;
    }
    return rc ? rc : (int)ej;
}

// The outermost levels: halve while the block is too large for the sweep to pay, then sweep
// (or recurse on one stream, for small blocks).
template <typename T> int potrf_top(bool lower, int64_t off, int64_t dim, T *A, int64_t lda, int *info, void *stream) {
    const int64_t W = potrf_panel<T>(dim);
    if (W > 0 && W < dim) return potrf_ahead<T>(lower, off, dim, W, A, lda, info, static_cast<hipStream_t>(stream));
    if (W != HALVE) return potrf_run<T>(lower, off, dim, A, lda, info, stream);
    T *D = A + off + off * lda;
    const int64_t n1 = ((dim / 2 + 255) / 256) * 256, n2 = dim - n1;
    int rc;
    if ((rc = potrf_top<T>(lower, off, n1, A, lda, info, stream))) return rc;
    T *P = lower ? D + n1 : D + n1 * lda;
    T *D2 = D + n1 + n1 * lda;
    if (lower) {
        if ((rc = trsm_impl<T>('R', 'L', 'T', 'N', n2, n1, T(1), D, lda, P, lda, stream))) return rc;
        if ((rc = syrk_call('L', 'N', n2, n1, T(-1), P, lda, T(1), D2, lda, stream))) return rc;
    } else {
        if ((rc = trsm_impl<T>('L', 'U', 'T', 'N', n1, n2, T(1), D, lda, P, lda, stream))) return rc;
        if ((rc = syrk_call('U', 'T', n2, n1, T(-1), P, lda, T(1), D2, lda, stream))) return rc;
    }
    return potrf_top<T>(lower, off + n1, n2, A, lda, info, stream);
}

template <typename T> int potrf_impl(char uplo, int64_t n, T *A, int64_t lda, int *info, void *stream) {
    const bool lower = (uplo == 'L' || uplo == 'l'), upper = (uplo == 'U' || uplo == 'u');
    if (!lower && !upper) return -1;
    if (n < 0 || n > DIM_MAX) return -2;
    if (n > 0 && !A) return -3;
    if (lda < max64(1, n)) return -4;
    if (!info) return -5;
    hipLaunchKernelGGL(clear_info_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream), info);
    const int rc = (int)hipGetLastError();
    if (rc || n == 0) return rc;
    return potrf_top<T>(lower, 0, n, A, lda, info, stream);
}

// ---------------------------------------------------------------------------
// Symmetric matrix product  C := alpha A B + beta C  (side L)  or  alpha B A + beta C  (side R),
// A symmetric, given by one triangle.  C is scaled by beta first; then A is halved recursively:
// the stored off-diagonal block couples the halves through two GEMMs (once as it is, once
// transposed), the diagonal blocks recurse, and diagonal blocks of order <= NB go to the kernel
// below, which mirrors the stored triangle into a full block in LDS and accumulates with the rows
// of the result across the lanes of a wave, like the triangular kernels.
// ---------------------------------------------------------------------------
template <typename T> struct SymmBlockArgs {
    const T *A;      // top-left element of the diagonal block
    int64_t lda;
    const T *B;      // the block's rows (side L) or columns (side R) of B
    int64_t ldb;
    T *C;            // the same part of C
    int64_t ldc;
    int nbk, nrhs, left, stored_lower;
    T alpha;
};

template <typename T> __global__ void __launch_bounds__(64 * WAVES) symm_block_kernel(const SymmBlockArgs<T> a) {
    using M = Mma16<T>;
    using acc_t = typename M::acc_t;
    __shared__ T e_cols[NB * NB];            // the full symmetric block, element (r, c) at [c * NB + r]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lc = lane & 15, lk = lane >> 4;
    const int nbk = a.nbk;
    const int lowr = a.stored_lower ? 1 : 0;
    constexpr int PER = NB / WAVES;

    // column operands of the matrix instruction: step s supplies element (4 s + lk) of right-hand side q
    const int q = (blockIdx.x * WAVES + wave) * MMA_RHS + lc;
    const int64_t bq = a.left ? a.ldb : 1, bx = a.left ? 1 : a.ldb;      // strides between / inside right-hand sides
    const int64_t cq = a.left ? a.ldc : 1, cx = a.left ? 1 : a.ldc;
    T xb[NB / 4];
#pragma unroll
    for (int sx = 0; sx < NB / 4; ++sx) {
        const int row = 4 * sx + lk;
        const bool in = q < a.nrhs && row < nbk;
        const T v = a.B[in ? (int64_t)row * bx + (int64_t)q * bq : 0];
        xb[sx] = in ? v : T(0);
    }
    // thread (wave w, lane t): stored row t, stored columns s = w, w + 4, ...; the referenced triangle
    // with its diagonal; everything else counts as zero here and is supplied by the mirror image
    T row[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int s = wave + u * WAVES;
        const int inside = (int)(lane < nbk) & (int)(s < nbk) & ((lowr & (int)(lane >= s)) | ((lowr ^ 1) & (int)(lane <= s)));
        const T v = a.A[(inside ? lane : 0) + (int64_t)(inside ? s : 0) * a.lda];
        row[u] = inside ? v : T(0);
    }
    for (int i = tid; i < NB * NB; i += 64 * WAVES) e_cols[i] = T(0);
    __syncthreads();
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int s = wave + u * WAVES;
        const int inside = (int)(lane < nbk) & (int)(s < nbk) & ((lowr & (int)(lane >= s)) | ((lowr ^ 1) & (int)(lane <= s)));
        if (inside) {
            e_cols[s * NB + lane] = row[u];
            e_cols[lane * NB + s] = row[u];
        }
    }
    __syncthreads();
    if ((blockIdx.x * WAVES + wave) * MMA_RHS >= a.nrhs) return;

    acc_t acc[NB / 16];
#pragma unroll
    for (int t = 0; t < NB / 16; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[t][r] = T(0);
#pragma unroll
    for (int sx = 0; sx < NB / 4; ++sx) {
        if (4 * sx < nbk) {                              // workgroup-uniform: columns past the order are zero
#pragma unroll
            for (int t = 0; t < NB / 16; ++t) acc[t] = M::mma(e_cols[(4 * sx + lk) * NB + 16 * t + lc], xb[sx], acc[t]);
        }
    }
    if (q < a.nrhs) {
#pragma unroll
        for (int t = 0; t < NB / 16; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int rr = 16 * t + M::drow(lane, r);
                if (rr < nbk) {
                    T *c = a.C + (int64_t)rr * cx + (int64_t)q * cq;
                    *c += a.alpha * acc[t][r];
                }
            }
    }
}

template <typename T> struct Symm {
    bool left, lower;
    const T *A;
    int64_t lda;
    const T *B;
    int64_t ldb;
    T *C;
    int64_t ldc, m, n;
    T alpha;
    void *stream;

    // Orders from 2 WIDE to FLAT_MAX, flat: with the block cut into diagonal blocks of order WIDE,
    // everything strictly below the block diagonal is one product whose depth per tile ends where the
    // tile's diagonal block begins, everything strictly above it one product whose depth starts where
    // that block ends (the stored triangle read as it is for one of them, transposed for the other),
    // and the diagonal blocks, which do not depend on each other, are one launch of the block
    // kernel.  Three launches in place of a recursion whose lower levels are small products.  Above
    // FLAT_MAX the recursion's full-depth products are the faster ones (measured at 16384).
    static constexpr int64_t FLAT_MAX = 8192;
    int flat(int64_t off, int64_t dim) const {
        const T *Ad = A + off + off * lda;
        const T *Bd = left ? B + off : B + off * ldb;
        T *Cd = left ? C + off : C + off * ldc;
        const int64_t mm = left ? dim : m, nn = left ? n : dim;
        // The first pass needs the entries (i, k), k < i, on the left (the stored triangle of a lower
        // matrix as it is) and the entries (k, j), k < j, on the right (the same triangle transposed);
        // the second pass the other way round.
        const char p1 = (left == lower) ? 'N' : 'T', p2 = p1 == 'N' ? 'T' : 'N';
        int rc = left ? xg::gemm_cut(p1, 'N', mm, nn, dim, alpha, Ad, lda, Bd, ldb, Cd, ldc, stream, 1, 0, (int)WIDE)
                      : xg::gemm_cut('N', p1, mm, nn, dim, alpha, Bd, ldb, Ad, lda, Cd, ldc, stream, 1, 1, (int)WIDE);
        if (rc == (int)hipErrorInvalidValue) return -1;   // not a shape for that kernel path; nothing was enqueued
        if (rc) return rc;
        rc = left ? xg::gemm_cut(p2, 'N', mm, nn, dim, alpha, Ad, lda, Bd, ldb, Cd, ldc, stream, 2, 0, (int)WIDE)
                  : xg::gemm_cut('N', p2, mm, nn, dim, alpha, Bd, ldb, Ad, lda, Cd, ldc, stream, 2, 1, (int)WIDE);
        if (rc) return rc;
        WideProdArgs<T> w;
        w.A = Ad;
        w.lda = lda;
        w.X = Bd;
        w.ldx = ldb;
        w.Y = Cd;
        w.ldy = ldc;
        w.dim = 0;
        w.nrhs = (int)(left ? n : m);
        w.left = left ? 1 : 0;
        w.etrans = 0;
        w.stored_lower = lower ? 1 : 0;
        w.unit = 0;
        w.alpha = alpha;
        w.batch_order = (int)dim;
        return launch_wide_product<T, 2>(w, stream);
    }

    int run(int64_t off, int64_t dim) const {
        if (dim >= 2 * WIDE && dim <= FLAT_MAX) {
            const int rc = flat(off, dim);
            if (rc != -1) return rc;                      // -1: take the recursion instead
        }
        if (dim > NB && dim <= WIDE) {
            WideProdArgs<T> w;
            w.A = A + off + off * lda;
            w.lda = lda;
            w.X = left ? B + off : B + off * ldb;
            w.ldx = ldb;
            w.Y = left ? C + off : C + off * ldc;
            w.ldy = ldc;
            w.dim = (int)dim;
            w.nrhs = (int)(left ? n : m);
            w.left = left ? 1 : 0;
            w.etrans = 0;
            w.stored_lower = lower ? 1 : 0;
            w.unit = 0;
            w.alpha = alpha;
            w.batch_order = 0;
            return launch_wide_product<T, 2>(w, stream);
        }
        if (dim <= NB) {
            SymmBlockArgs<T> a;
            a.A = A + off + off * lda;
            a.lda = lda;
            a.B = left ? B + off : B + off * ldb;
            a.ldb = ldb;
            a.C = left ? C + off : C + off * ldc;
            a.ldc = ldc;
            a.nbk = (int)dim;
            a.nrhs = (int)(left ? n : m);
            a.left = left ? 1 : 0;
            a.stored_lower = lower ? 1 : 0;
            a.alpha = alpha;
            constexpr int PER_WG = MMA_RHS * WAVES;
            hipLaunchKernelGGL(symm_block_kernel<T>, dim3((unsigned)((a.nrhs + PER_WG - 1) / PER_WG)), dim3(64 * WAVES), 0,
                               static_cast<hipStream_t>(stream), a);
            return (int)hipGetLastError();
        }
        const int64_t n1 = ((dim / 2 + NB - 1) / NB) * NB, n2 = dim - n1, o2 = off + n1;
        // stored off-diagonal block: A21 (n2 x n1) of a lower, A12 (n1 x n2) of an upper triangle
        const T *S = lower ? A + o2 + off * lda : A + off + o2 * lda;
        const char as12 = lower ? 'T' : 'N', as21 = lower ? 'N' : 'T';   // how S gives A12 and A21
        int rc;
        if (left) {
            if ((rc = real_gemm<T>(as12, 'N', n1, n, n2, alpha, S, lda, B + o2, ldb, T(1), C + off, ldc, stream))) return rc;
            if ((rc = real_gemm<T>(as21, 'N', n2, n, n1, alpha, S, lda, B + off, ldb, T(1), C + o2, ldc, stream))) return rc;
        } else {
            if ((rc = real_gemm<T>('N', as21, m, n1, n2, alpha, B + o2 * ldb, ldb, S, lda, T(1), C + off * ldc, ldc, stream)))
                return rc;
            if ((rc = real_gemm<T>('N', as12, m, n2, n1, alpha, B + off * ldb, ldb, S, lda, T(1), C + o2 * ldc, ldc, stream)))
                return rc;
        }
        if ((rc = run(off, n1))) return rc;
        return run(o2, n2);
    }
};

template <typename T>
int symm_impl(char side, char uplo, int64_t m, int64_t n, T alpha, const T *A, int64_t lda, const T *B, int64_t ldb,
              T beta, T *C, int64_t ldc, void *stream) {
    const bool left = (side == 'L' || side == 'l'), right = (side == 'R' || side == 'r');
    const bool lower = (uplo == 'L' || uplo == 'l'), upper = (uplo == 'U' || uplo == 'u');
    if (!left && !right) return -1;
    if (!lower && !upper) return -2;
    if (m < 0 || m > DIM_MAX) return -3;
    if (n < 0 || n > DIM_MAX) return -4;
    const bool ab_read = alpha != T(0) && m > 0 && n > 0;
    if (ab_read && !A) return -6;
    if (lda < max64(1, left ? m : n)) return -7;
    if (ab_read && !B) return -8;
    if (ldb < max64(1, m)) return -9;
    if (m > 0 && n > 0 && !C) return -11;
    if (ldc < max64(1, m)) return -12;
    if (m == 0 || n == 0) return 0;
    if (!ab_read && beta == T(1)) return 0;
    if (beta != T(1)) {
        const int rc = scale_b<T>(C, ldc, m, n, beta, stream);
        if (rc) return rc;
    }
    if (!ab_read) return 0;
    Symm<T> s{left, lower, A, lda, B, ldb, C, ldc, m, n, alpha, stream};
    return s.run(0, left ? m : n);
}

}  // namespace

namespace xg {
void reset_l3_tuning() {
    t_potrf_panel = -1;
    t_potrf_block = 256;
}
}  // namespace xg

extern "C" {

int xgemm_dsymm(char side, char uplo, int64_t m, int64_t n, double alpha, const double *A, int64_t lda, const double *B,
                int64_t ldb, double beta, double *C, int64_t ldc, void *stream) {
    return symm_impl<double>(side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc, stream);
}

int xgemm_ssymm(char side, char uplo, int64_t m, int64_t n, float alpha, const float *A, int64_t lda, const float *B,
                int64_t ldb, float beta, float *C, int64_t ldc, void *stream) {
    return symm_impl<float>(side, uplo, m, n, alpha, A, lda, B, ldb, beta, C, ldc, stream);
}

int xgemm_release_thread_resources(void) { return release_side_lanes(); }

int xgemm_force_potrf_panel(int64_t width) {
    if (width < -1 || width > DIM_MAX) return -1;
    t_potrf_panel = width;
    return 0;
}

int xgemm_force_potrf_block(int order) {
    if (order != -1 && order != 64 && order != 128 && order != 256) return -1;
    t_potrf_block = order < 0 ? 256 : order;
    return 0;
}

int xgemm_dpotrf(char uplo, int64_t n, double *A, int64_t lda, int *info, void *stream) {
    return potrf_impl<double>(uplo, n, A, lda, info, stream);
}

int xgemm_spotrf(char uplo, int64_t n, float *A, int64_t lda, int *info, void *stream) {
    return potrf_impl<float>(uplo, n, A, lda, info, stream);
}

int xgemm_dtrmm(char side, char uplo, char transa, char diag, int64_t m, int64_t n, double alpha, const double *A,
                int64_t lda, double *B, int64_t ldb, void *stream) {
    return trmm_impl<double>(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb, stream);
}

int xgemm_strmm(char side, char uplo, char transa, char diag, int64_t m, int64_t n, float alpha, const float *A,
                int64_t lda, float *B, int64_t ldb, void *stream) {
    return trmm_impl<float>(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb, stream);
}

int xgemm_dtrsm(char side, char uplo, char transa, char diag, int64_t m, int64_t n, double alpha, const double *A,
                int64_t lda, double *B, int64_t ldb, void *stream) {
    return trsm_impl<double>(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb, stream);
}

int xgemm_strsm(char side, char uplo, char transa, char diag, int64_t m, int64_t n, float alpha, const float *A,
                int64_t lda, float *B, int64_t ldb, void *stream) {
    return trsm_impl<float>(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb, stream);
}

}  // extern "C"
