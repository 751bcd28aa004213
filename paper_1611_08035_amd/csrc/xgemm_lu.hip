// xgemm_lu.hip -- LU factorisation with partial pivoting on the level-3 routines (the other
// LAPACK-level driver the paper names as resting on GEMM, Abstract and Sec. 1).
//
//     P A = L U,   A m x n,  L unit lower trapezoidal, U upper trapezoidal, both in place;
//     ipiv[j] (1-based) is the row that was interchanged with row j at step j.
//
// Organisation.  The matrix is halved recursively by columns (left half; triangular solve and product
// for the right half; right half), so that all arithmetic except that of the base panels runs in the
// solve and product kernels at the greatest depth there is.  A base panel (at most 128 columns) is
//   - where exchange memory is at hand (the caller's, xgemm_*getrf_ws, or the buffer the library allocates
//     per device on the first call outside a stream capture) or the panel has at most 128 rows: factored by
//     all the workgroups its rows need at once, each holding a stripe of rows in LDS, the pivot of a column
//     agreed through the exchange memory (getrf_coop_kernel; the only kernel of the library in which a
//     workgroup waits for another, which is why such factorisations are ordered one behind the other on a
//     device, see getrf_impl);
//   - otherwise (a captured call without a buffer, a panel taller than the device has compute units for):
//     halved further down to leaves of up to LEAF columns, each factored by ONE workgroup (getf2_kernel):
//     the search for the pivot is a reduction inside the workgroup, a leaf costs one launch, not one per
//     column, and carries its interchanges through the columns of its base panel.  Two leaves side by side
//     run without a launch between them: the left one also solves for the block row of U above the right
//     one, the right one applies the left one's update as it loads.
// A base panel's interchanges are applied to the other columns of every enclosing half by laswp_kernel.
#include "../../include/xgemm.h"
#include "../../include/xgemm_tuning.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <type_traits>

namespace {

inline int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }
inline int64_t min64(int64_t a, int64_t b) { return a < b ? a : b; }
constexpr int64_t DIM_MAX = 0x7fffffff;
constexpr int LEAF = 8;          // most columns one workgroup factors by itself
constexpr int LEAF_NT = 512;     // its threads (two waves per SIMD, so that each thread may hold 64 elements in registers)
constexpr int LEAF_WAVES = LEAF_NT / 64;
// elements of the leaf per thread, ROWS x W with W = 8, 4, 2 or 1 columns: what the registers of a lane hold
// beside the rest of the kernel's state
template <typename T> constexpr int leaf_elems(int w) { return sizeof(T) == 8 ? (w == 2 ? 40 : 48) : (w == 2 ? 56 : 64); }

thread_local int64_t t_lu_panel = -1;   // -1: by the order; W > 0: panels of W columns
thread_local int t_lu_shared = -1;       // -1: shared panels wherever they can be used; 0: leaves of one workgroup only
// First look of a poll put off by this many 64-clock sleeps.  While headers and rows were published right before
// they were polled for, a look that came too early cost a whole round trip more and 18 resp. 13 sleeps paid
// (52.5 -> 48.1 ms at 8192); since both are published a barrier ahead of the poll, no delay is best.
constexpr int LU_HDR_DELAY = 0, LU_ROW_DELAY = 0;
thread_local int t_lu_hdr_delay = LU_HDR_DELAY, t_lu_row_delay = LU_ROW_DELAY;
thread_local int t_lu_spin_limit = 1 << 18;   // polls a workgroup of a shared panel waits for the others (about a microsecond each)

template <typename T> __device__ __forceinline__ T abs_of(T x) { return x < T(0) ? -x : x; }

// `count` elements from `base` on as a buffer: an element offset at or beyond count reads as zero and is not
// written, so that the rows of a leaf past the end of the matrix need no branch (and no wait that a branch
// per access brings with it).
template <typename T> struct Rows {
    __amdgpu_buffer_rsrc_t rsrc;
    __device__ __forceinline__ Rows(T *base, int count)
        : rsrc(__builtin_amdgcn_make_buffer_rsrc(base, 0, count > 0 ? count * (int)sizeof(T) : 0, 0x00020000)) {}
    __device__ __forceinline__ T get(int at) const {
        if constexpr (sizeof(T) == 8) {
            typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
            return __builtin_bit_cast(T, (u32x2)__builtin_amdgcn_raw_buffer_load_b64(rsrc, at * (int)sizeof(T), 0, 0));
        } else {
            return __builtin_bit_cast(T, (unsigned int)__builtin_amdgcn_raw_buffer_load_b32(rsrc, at * (int)sizeof(T), 0, 0));
        }
    }
    __device__ __forceinline__ void put(int at, T v) const {
        if constexpr (sizeof(T) == 8) {
            typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, v), rsrc, at * (int)sizeof(T), 0, 0);
        } else {
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, v), rsrc, at * (int)sizeof(T), 0, 0);
        }
    }
};
// smallest magnitude whose reciprocal is finite and normal (LAPACK's safe minimum)
template <typename T> struct RcpLimit;
template <> struct RcpLimit<double> { static __device__ __forceinline__ double tiny() { return 2.2250738585072014e-308; } };
template <> struct RcpLimit<float> { static __device__ __forceinline__ float tiny() { return 1.17549435e-38f; } };

// Candidate for the pivot: the largest magnitude, and among equal magnitudes the smallest row.
template <typename T> struct Cand {
    T val;
    int row;
};
template <typename T> __device__ __forceinline__ Cand<T> better(Cand<T> a, Cand<T> b) {
    return (b.val > a.val || (b.val == a.val && b.row < a.row)) ? b : a;
}
// A candidate as another lane holds it, the lanes paired by a data-parallel-primitive pattern (register moves
// between lanes of a row of 16, no LDS round trip): 0xB1 and 0x4E exchange neighbours inside a quad (lane ^ 1,
// lane ^ 2), 0x141 mirrors each half row (lane i <-> 7 - i), 0x140 each row (i <-> 15 - i).
template <int CTRL> __device__ __forceinline__ int dpp_word(int v) { return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false); }
template <int CTRL, typename T> __device__ __forceinline__ Cand<T> dpp_cand(Cand<T> c) {
    Cand<T> o;
    if constexpr (sizeof(T) == 8) {
        typedef int i32x2 __attribute__((ext_vector_type(2)));
        i32x2 p = __builtin_bit_cast(i32x2, c.val);
        p[0] = dpp_word<CTRL>(p[0]);
        p[1] = dpp_word<CTRL>(p[1]);
        o.val = __builtin_bit_cast(T, p);
    } else {
        o.val = __builtin_bit_cast(T, dpp_word<CTRL>(__builtin_bit_cast(int, c.val)));
    }
    o.row = dpp_word<CTRL>(c.row);
    return o;
}
template <typename T> __device__ __forceinline__ Cand<T> lane_cand(Cand<T> c, int lane) {
    Cand<T> o;
    if constexpr (sizeof(T) == 8) {
        typedef int i32x2 __attribute__((ext_vector_type(2)));
        i32x2 p = __builtin_bit_cast(i32x2, c.val);
        p[0] = __builtin_amdgcn_readlane(p[0], lane);
        p[1] = __builtin_amdgcn_readlane(p[1], lane);
        o.val = __builtin_bit_cast(T, p);
    } else {
        o.val = __builtin_bit_cast(T, __builtin_amdgcn_readlane(__builtin_bit_cast(int, c.val), lane));
    }
    o.row = __builtin_amdgcn_readlane(c.row, lane);
    return o;
}
// The best candidate of the wave, in every lane.  `better` picks the same winner whichever way round two
// different candidates are given, so after each pairing both partners hold it: four pairings make every row of 16
// lanes agree, and the four rows are compared as scalars.
template <typename T> __device__ __forceinline__ Cand<T> wave_best(Cand<T> c) {
    c = better(c, dpp_cand<0xB1>(c));
    c = better(c, dpp_cand<0x4E>(c));
    c = better(c, dpp_cand<0x141>(c));
    c = better(c, dpp_cand<0x140>(c));
    return better(better(lane_cand(c, 0), lane_cand(c, 16)), better(lane_cand(c, 32), lane_cand(c, 48)));
}

// ---------------------------------------------------------------------------
// Row interchanges, a batch at a time.  The interchanges k = 0 .. cnt - 1 (row top + k with row piv[k], in that
// order, cnt <= G) touch at most 2 G rows and permute them the same way in every column, so the permutation is
// worked out once per batch and workgroup, and a thread then moves its column with loads and stores that do not
// depend on each other, instead of a chain of cnt dependent exchanges.
//   slots 0 .. G-1 stand for the rows top + k, slots G .. 2G-1 for the rows piv[k]; a row that occurs several
//   times is represented by its first slot (canon); lane j of the first wave follows the content that started in
//   slot j through the interchanges, which gives each slot the slot its final content comes from (src).
// LDS: rows[2G], canon[2G], src[2G] ints and vals[2G][NTHR] elements.  Every thread of the workgroup must call
// (barriers inside); a thread without a column passes col == nullptr.
// ---------------------------------------------------------------------------
template <typename T, int G, int NTHR> struct SwapLds {
    int rows[2 * G], canon[2 * G], src[2 * G];
    T vals[2 * G][NTHR];
};
template <typename T, int G, int NTHR>
__device__ __forceinline__ void swap_batch(SwapLds<T, G, NTHR> &L, T *col, int top, const int *piv, int piv_bias, int cnt,
                                           int tid) {
    static_assert(2 * G <= 64, "the slots are the lanes of one wave");
    if (tid < 2 * G) {
        const int k = tid < G ? tid : tid - G;
        L.rows[tid] = k < cnt ? (tid < G ? top + k : piv[k] + piv_bias) : -1 - tid;   // unused slots: distinct, never a row
    }
    __syncthreads();
    if (tid < 2 * G) {
        int c = tid;
        for (int j = tid - 1; j >= 0; --j)
            if (L.rows[j] == L.rows[tid]) c = j;
        L.canon[tid] = c;
    }
    __syncthreads();
    if (tid < 2 * G) {
        // lane j follows the content that started in slot j through the interchanges: no lane needs another's state
        int pos = tid;
        for (int k = 0; k < cnt; ++k) {
            const int a = L.canon[k], b = L.canon[G + k];
            pos = pos == a ? b : (pos == b ? a : pos);
        }
        L.src[tid] = -1;
        __builtin_amdgcn_wave_barrier();
        if (L.canon[tid] == tid && L.rows[tid] >= 0) L.src[pos] = tid;
    }
    __syncthreads();
    if (col) {
        T v[2 * G];
#pragma unroll
        for (int j = 0; j < 2 * G; ++j) v[j] = L.src[j] >= 0 ? col[L.rows[j]] : T(0);
#pragma unroll
        for (int j = 0; j < 2 * G; ++j) L.vals[j][tid % NTHR] = v[j];
#pragma unroll 4
        for (int j = 0; j < 2 * G; ++j) {
            const int sj = L.src[j];
            if (sj >= 0 && sj != j) col[L.rows[j]] = L.vals[sj][tid % NTHR];
        }
    }
    __syncthreads();
}

// Columns [j0, j0 + w) of A, rows j0 .. m - 1, w <= W: Gaussian elimination with partial pivoting, one column
// at a time, by one workgroup.  Row j0 + t + q * LEAF_NT belongs to thread t for the whole leaf.
// RESIDENT: the leaf fits the registers (at most LEAF_NT * ROWS rows, ROWS x W = 64 elements per thread): it is
// loaded once and stored once.  Otherwise it stays in memory (the caches of this CU) and every column is one
// pass over the rows below it, ROWS rows of a thread at a time.
// Per column c (row r = j0 + c), with ONE barrier:
//   - every thread knows the largest entry among its own rows (found while the column before was updated);
//     a reduction over each wave picks the wave's candidate (largest magnitude, smallest row among equals),
//     and the lane that owns it leaves the whole candidate row (all w columns) in LDS, as thread c does
//     with row r;
//   - barrier; every thread reduces the waves' candidates alike, so all know the pivot row p, its values U and
//     the old row r without reading either from memory;
//   - rows r and p change places: the owner of r takes U, the owner of p takes the old row r (no other thread
//     touches either row);
//   - the column is divided by the pivot (times its reciprocal; no multiplier exceeds one), the columns to
//     its right inside the leaf are updated, and the search for the next pivot rides on that pass.
// The LDS slots alternate with the parity of c, so that a wave that is a column ahead does not overwrite what
// a slower one still reads.  At the end the leaf's interchanges are carried through the other columns of the
// enclosing panel [c_lo, c_hi) in one batch.  A zero pivot is recorded in *info (first one only, 1-based
// column) and its column left as it is.  ipiv[j0 + c] receives the pivot's row + 1.
template <typename T, int ROWS, int W, bool RESIDENT>
__global__ void __launch_bounds__(LEAF_NT) getf2_kernel(T *A, int64_t lda, int m, int j0, int w, int c_lo, int c_hi,
                                                        int *ipiv, int *info, int pre, int post) {
    __shared__ T s_val[2][LEAF_WAVES];
    __shared__ int s_row[2][LEAF_WAVES];
    __shared__ T s_cand[2][LEAF_WAVES][W];
    __shared__ T s_top[2][W];
    __shared__ int s_piv[LEAF];
    __shared__ SwapLds<T, LEAF, 128> s_swap;
    constexpr int NONE = 0x7fffffff;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    T *const P = A + (int64_t)j0 * lda;          // column j0 of the matrix
    __shared__ T s_pair[LEAF][LEAF];             // pre: the block row of U above this leaf; post: the leaf's own L11
    T a[ROWS][W];
    Cand<T> mine{T(-1), NONE};
    // pre > 0 (resident leaves only): the `pre` columns left of this leaf are its factored left sibling, whose
    // update of these columns is still due: rows j0 - pre .. j0 - 1 of these columns hold U12 (the sibling left it
    // there, see post below) and every row from j0 on takes  a -= L21 U12  as it is loaded.
    if (RESIDENT && W > 1 && pre > 0) {       // (leaves of one column are not paired: they have no register to spare)
        if (tid < LEAF * LEAF) {
            const int u = tid / LEAF, d = tid % LEAF;
            s_pair[u][d] = (u < pre && d < w) ? A[(j0 - pre + u) + (int64_t)(j0 + d) * lda] : T(0);
        }
        __syncthreads();
    }
    if (RESIDENT) {
        // all loads of the leaf are issued before anything looks at them
#pragma unroll
        for (int d = 0; d < W; ++d) {
            const Rows<T> col(P + j0 + (int64_t)d * lda, d < w ? m - j0 : 0);      // columns past w: all zeros
#pragma unroll
            for (int q = 0; q < ROWS; ++q) a[q][d] = col.get(tid + q * LEAF_NT);
        }
        if (W > 1 && pre > 0) {
            // one column of the sibling's L at a time, HALF rows of a thread in flight together
            constexpr int HALF = ROWS > 16 ? 8 : (ROWS + 1) / 2;
            for (int u = 0; u < pre; ++u) {
                const Rows<T> lcol(P + j0 + (int64_t)(u - pre) * lda, m - j0);
#pragma unroll
                for (int h = 0; h < ROWS; h += HALF) {
                    T l[HALF];
#pragma unroll
                    for (int q = h; q < h + HALF && q < ROWS; ++q) l[q - h] = lcol.get(tid + q * LEAF_NT);
#pragma unroll
                    for (int q = h; q < h + HALF && q < ROWS; ++q)
#pragma unroll
                        for (int d = 0; d < W; ++d) a[q][d] = a[q][d] - l[q - h] * s_pair[u][d];
                }
            }
        }
#pragma unroll
        for (int q = 0; q < ROWS; ++q) {
            const int i = j0 + tid + q * LEAF_NT;
            if (i < m) {
                const T v = abs_of(a[q][0]);
                if (v > mine.val) { mine.val = v; mine.row = i; }
            }
        }
    } else {
        for (int i = j0 + tid; i < m; i += LEAF_NT) {
            const T v = abs_of(P[i]);
            if (v > mine.val) { mine.val = v; mine.row = i; }
        }
    }
    for (int c = 0; c < w; ++c) {
        const int r = j0 + c, buf = c & 1;
        const Cand<T> wb = wave_best(mine);
        if (wb.row == NONE) {
            if (lane == 0) { s_val[buf][wave] = T(-1); s_row[buf][wave] = NONE; }
        } else if (mine.row == wb.row) {          // one lane: rows are distinct
            s_val[buf][wave] = wb.val;
            s_row[buf][wave] = wb.row;
            if (RESIDENT) {
                const int qc = (wb.row - j0) / LEAF_NT;
#pragma unroll
                for (int q = 0; q < ROWS; ++q)
                    if (q == qc) {
#pragma unroll
                        for (int d = 0; d < W; ++d) s_cand[buf][wave][d] = a[q][d];
                    }
            } else {
#pragma unroll
                for (int d = 0; d < W; ++d) s_cand[buf][wave][d] = d < w ? P[wb.row + (int64_t)d * lda] : T(0);
            }
        }
        if (tid == c) {                           // row r is this thread's first row
#pragma unroll
            for (int d = 0; d < W; ++d) s_top[buf][d] = RESIDENT ? a[0][d] : (d < w ? P[r + (int64_t)d * lda] : T(0));
        }
        __syncthreads();
        Cand<T> best{T(-1), NONE};
        int bw = 0;
#pragma unroll
        for (int v = 0; v < LEAF_WAVES; ++v) {
            const Cand<T> x{s_val[buf][v], s_row[buf][v]};
            if (x.val > best.val || (x.val == best.val && x.row < best.row)) { best = x; bw = v; }
        }
        const int p = best.row;
        T U[W], top[W];
#pragma unroll
        for (int d = 0; d < W; ++d) { U[d] = s_cand[buf][bw][d]; top[d] = s_top[buf][d]; }
        T pivot = T(0);
#pragma unroll
        for (int d = 0; d < W; ++d) pivot = (d == c) ? U[d] : pivot;
        // wave-uniform facts about the pivot, as scalars: what depends on them is branched over, not computed and
        // thrown away (a double-precision division costs some thirty instructions)
        const bool nonzero = __builtin_amdgcn_readfirstlane((int)(pivot != T(0))) != 0;
        // the column is scaled by the reciprocal of the pivot, as LAPACK does (one division per column instead of
        // one per row; |a| <= |pivot| still gives |a * (1 / pivot)| <= 1 after rounding), unless the reciprocal
        // would overflow
        const bool by_rcp = __builtin_amdgcn_readfirstlane((int)(abs_of(pivot) >= RcpLimit<T>::tiny())) != 0;
        const T rcp = by_rcp ? T(1) / pivot : T(0);
        if (tid == 0) {
            ipiv[r] = p + 1;
            s_piv[c] = p;
            if (!nonzero && *info == 0) *info = r + 1;
        }
        const bool exchange = nonzero && p != r;
        mine.val = T(-1);
        mine.row = NONE;
        if (RESIDENT) {
            if (exchange) {
                const int tp = (p - j0) % LEAF_NT, qp = (p - j0) / LEAF_NT;
                if (tid == c) {
#pragma unroll
                    for (int d = 0; d < W; ++d) a[0][d] = U[d];
                }
                if (tid == tp) {
#pragma unroll
                    for (int q = 0; q < ROWS; ++q)
                        if (q == qp) {
#pragma unroll
                            for (int d = 0; d < W; ++d) a[q][d] = top[d];
                        }
                }
            }
            // the update of the rows below r, with the column index as a compile-time constant inside each case so
            // that every register of the leaf is addressed statically
            auto update = [&](auto c_tag) {
                constexpr int C = decltype(c_tag)::value;
#pragma unroll
                for (int q = 0; q < ROWS; ++q) {
                    const int i = j0 + tid + q * LEAF_NT;
                    if (i > r && i < m) {
                        T l = a[q][C];
                        if (nonzero) {
                            if (by_rcp) l = l * rcp;
                            else l = l / pivot;
                        }
                        a[q][C] = l;
#pragma unroll
                        for (int d = C + 1; d < W; ++d)
                            if (d < w) a[q][d] = a[q][d] - l * U[d];
                        if constexpr (C + 1 < W) {
                            if (C + 1 < w) {
                                const T v = abs_of(a[q][C + 1]);
                                if (v > mine.val) { mine.val = v; mine.row = i; }
                            }
                        }
                    }
                }
            };
            switch (c) {
                case 0: update(std::integral_constant<int, 0>{}); break;
                case 1: if constexpr (W > 1) update(std::integral_constant<int, 1>{}); break;
                case 2: if constexpr (W > 2) update(std::integral_constant<int, 2>{}); break;
                case 3: if constexpr (W > 3) update(std::integral_constant<int, 3>{}); break;
                case 4: if constexpr (W > 4) update(std::integral_constant<int, 4>{}); break;
                case 5: if constexpr (W > 5) update(std::integral_constant<int, 5>{}); break;
                case 6: if constexpr (W > 6) update(std::integral_constant<int, 6>{}); break;
                default: if constexpr (W > 7) update(std::integral_constant<int, 7>{}); break;
            }
        } else {
            if (exchange && tid == c) {
#pragma unroll
                for (int d = 0; d < W; ++d)
                    if (d < w) P[r + (int64_t)d * lda] = U[d];
            }
            for (int i0 = j0 + tid; i0 < m; i0 += ROWS * LEAF_NT) {
                T x[ROWS][W];
#pragma unroll
                for (int q = 0; q < ROWS; ++q) {
                    const int i = i0 + q * LEAF_NT;
                    const bool live = i > r && i < m, moved = exchange && i == p;
#pragma unroll
                    for (int d = 0; d < W; ++d)
                        x[q][d] = moved ? top[d] : ((live && d >= c && d < w) ? P[i + (int64_t)d * lda] : T(0));
                }
#pragma unroll
                for (int q = 0; q < ROWS; ++q) {
                    const int i = i0 + q * LEAF_NT;
                    const bool live = i > r && i < m, moved = exchange && i == p;
                    if (!live) continue;
                    T l = T(0);
#pragma unroll
                    for (int d = 0; d < W; ++d) l = (d == c) ? x[q][d] : l;
                    if (nonzero) {
                        if (by_rcp) l = l * rcp;
                        else l = l / pivot;
                    }
#pragma unroll
                    for (int d = 0; d < W; ++d) {
                        if (d >= w) continue;
                        T *const dst = P + i + (int64_t)d * lda;
                        if (d < c) {
                            if (moved) *dst = x[q][d];          // the part of the old row r left of column c moves too
                        } else if (d == c) {
                            if (nonzero || moved) *dst = l;
                        } else {
                            const T y = x[q][d] - l * U[d];
                            *dst = y;
                            if (d == c + 1) {
                                const T v = abs_of(y);
                                if (v > mine.val) { mine.val = v; mine.row = i; }
                            }
                        }
                    }
                }
            }
        }
    }
    // the leaf's interchanges in the other columns of the enclosing panel, 128 columns at a time; before the leaf
    // itself goes back to memory, so that these loads do not queue behind its stores
    const int outside = (c_hi - c_lo) - w;
    for (int x0 = 0; x0 < outside; x0 += 128) {       // uniform trip count; s_piv is complete after the first barrier inside
        const int x = x0 + tid;
        T *col = nullptr;
        if (tid < 128 && x < outside) col = A + (int64_t)(c_lo + x + (c_lo + x >= j0 ? w : 0)) * lda;
        swap_batch<T, LEAF, 128>(s_swap, col, j0, s_piv, 0, w, tid);
    }
    // post > 0 (resident leaves only): the `post` columns right of this leaf are its right sibling; their rows
    // j0 .. j0 + w - 1 (already interchanged above) become the block row  U12 = L11^-1 A12  here, one thread per
    // column, with L11 from the registers of the threads that own the leaf's first w rows, so that no solve has to
    // be launched between the two leaves
    if (RESIDENT && W > 1 && post > 0) {
        __syncthreads();                              // s_pair may still be read as U12 by a slow wave of the load
        if (tid < w) {
#pragma unroll
            for (int d = 0; d < W; ++d) s_pair[tid][d] = a[0][d];     // row j0 + tid is this thread's first row
        }
        __syncthreads();
        if (tid < post) {
            T *const x = A + j0 + (int64_t)(j0 + w + tid) * lda;
            T u[LEAF];
#pragma unroll
            for (int t = 0; t < LEAF; ++t) u[t] = t < w ? x[t] : T(0);
#pragma unroll
            for (int t = 1; t < LEAF; ++t)
#pragma unroll
                for (int d = 0; d < t; ++d)
                    if (t < w) u[t] = u[t] - s_pair[t][d] * u[d];
#pragma unroll
            for (int t = 1; t < LEAF; ++t)
                if (t < w) x[t] = u[t];
        }
    }
    // the leaf back to memory, a column at a time
    if (RESIDENT) {
#pragma unroll
        for (int d = 0; d < W; ++d) {
            const Rows<T> col(P + j0 + (int64_t)d * lda, d < w ? m - j0 : 0);      // columns past w: nothing is written
#pragma unroll
            for (int q = 0; q < ROWS; ++q) col.put(tid + q * LEAF_NT, a[q][d]);
        }
    }
}

// ---------------------------------------------------------------------------
// A panel shared by many workgroups.  The leaf above is one workgroup on one compute unit while the rest of
// the device waits; here the rows of a panel of up to NB columns are dealt to G workgroups in stripes of RPW
// rows, each workgroup keeps its stripe in LDS for the whole panel, and the one decision per column that
// concerns all of them, the pivot, is taken by every workgroup alike from G candidates exchanged through
// memory.  A workgroup has RPW * TPR computing threads (TPR threads per row, lanes of one wave) and one more
// wave, the communicator, that talks to the other workgroups while the computing waves work.  For column c
// (row r = j0 + c, sequence number r + 1):
//   - the communicator polls the G headers {magnitude, row, sequence number} of column c until all carry
//     this column's number, which gives the pivot row p to every workgroup alike (largest magnitude, smallest
//     row among equals), and fetches the row that p's owner published with its header and the row r that
//     workgroup 0 published, into LDS; meanwhile the computing waves are still applying the pivot of column
//     c - 1 to their stripe;                                                                        barrier B
//   - the stripe is up to date with column c - 1.  The communicator works out what all threads need of the
//     pivot (how to scale, the reciprocal), writes ipiv and info (workgroup 0), and then, for column c + 1,
//     from what the stripe WILL hold once pivot c is applied (computed with the very operations the computing
//     waves use, scaled() and eliminated(), so that the magnitudes it compares are those of the entries that
//     get stored): the stripe's candidate, which it publishes at once, then the candidate's whole row and
//     (workgroup 0) the row that will be row r + 1, which it publishes too;                          barrier C
//   - the computing waves apply pivot c: rows r and p change places inside the stripes that hold them, the
//     column is scaled, the columns on its right are updated, while the communicator is already polling
//     for column c + 1.
// So a column costs the other workgroups' store-to-load latency once (header and row travel together) plus
// what the communicator computes between the barriers, and the update of the stripe runs beside the exchange.
// Every published item is one aligned 16-byte store that carries the column's sequence number beside its
// value; a reader tells by itself whether what it read belongs to this column, so nothing waits for an
// acknowledgement.  The exchange memory is written through to memory and read around the caches (the L2s of
// different XCDs are not coherent with each other).  Slots alternate with the parity of c: whoever publishes
// for column c + 1 has seen every header of column c, whose owners had finished reading column c - 1.
// Sequence numbers are unique within a factorisation and the exchange memory is cleared when it starts, so a
// stale slot never matches.  Every wait is bounded: a communicator that does not see what it waits for
// within `spin_limit` polls raises a flag in the exchange memory and gives up; whoever sees the flag gives up
// too, and *info becomes -1.  The G workgroups must be resident together (one per compute unit: the host
// never asks for more than the device has).
// ---------------------------------------------------------------------------
constexpr int COOP_GMAX = 256;            // most workgroups that share a panel
constexpr int COOP_NB = 128;              // widest shared panel
constexpr size_t COOP_FLAG_BYTES = 256;   // the time-out flag (first word)
constexpr size_t COOP_HDR_BYTES = 2 * (size_t)COOP_GMAX * 16;
constexpr size_t COOP_ROW_BYTES = 2 * (size_t)COOP_NB * 16;                 // elements travel as {value, sequence number}
constexpr size_t COOP_BYTES = COOP_FLAG_BYTES + COOP_HDR_BYTES + (COOP_GMAX + 1) * COOP_ROW_BYTES;   // flag, headers, a candidate row per workgroup, row r
constexpr int THROUGH = 17;               // cache policy bits sc0 | sc1: system scope
constexpr int COOP_INFO_TIMEOUT = -1;

template <typename T> struct CoopCfg;
template <> struct CoopCfg<double> { static constexpr int RPW = 128, TPR = 4; };
template <> struct CoopCfg<float> { static constexpr int RPW = 128, TPR = 4; };

// the whole exchange memory to zero: no slot carries a sequence number of an earlier factorisation
__global__ void __launch_bounds__(256) coop_clear_kernel(uint4 *xch) {
    for (unsigned i = blockIdx.x * 256 + threadIdx.x; i < COOP_BYTES / 16; i += gridDim.x * 256) xch[i] = uint4{0u, 0u, 0u, 0u};
}

template <typename T, int RPW, int TPR>
__global__ void __launch_bounds__(RPW * TPR + 64) getrf_coop_kernel(T *A, int64_t lda, int m, int j0, int nb, int *ipiv, int *info,
                                                                    unsigned char *xch, int spin_limit, int hdr_delay, int row_delay) {
    static_assert(COOP_NB <= RPW, "row r must belong to workgroup 0 for every column of the panel");
    static_assert(64 % TPR == 0, "the threads of a row share a wave");
    constexpr int NTC = RPW * TPR;         // computing threads
    constexpr int NWC = NTC / 64;          // computing waves; wave NWC is the communicator
    constexpr int RW = 64 / TPR;           // rows per wave
    constexpr int LS = RPW + 1;            // odd column stride: a row is read without bank conflicts
    constexpr int NONE = 0x7fffffff;
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    extern __shared__ __align__(16) unsigned char coop_lds[];
    T *const P = reinterpret_cast<T *>(coop_lds);          // P[d * LS + i]: column d, local row i
    __shared__ T s_Ub[2][COOP_NB], s_topb[2][COOP_NB];      // pivot row and old row r, by the parity of the column
    __shared__ int s_p, s_abort, s_how;                     // s_how: 0 pivot is zero, 1 scale by s_rcp, 2 divide
    __shared__ T s_rcp;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool comm = wave == NWC;
    const int g = blockIdx.x, G = gridDim.x;
    const int i0 = j0 + g * RPW;                            // first row of this stripe
    const int nrows = (m - i0) < RPW ? (m - i0) : RPW;

    // exchange memory
    unsigned char *const x_hdr = xch + COOP_FLAG_BYTES;
    unsigned char *const x_top = x_hdr + COOP_HDR_BYTES;                   // [parity][column]
    unsigned char *const x_rows = x_top + COOP_ROW_BYTES;                  // [workgroup][parity][column]
    const __amdgpu_buffer_rsrc_t r_flag = __builtin_amdgcn_make_buffer_rsrc(xch, 0, 4, 0x00020000);

    // the stripe as one range-checked buffer: rows past the end of the matrix get an offset outside it (they read
    // as zero and are not written)
    constexpr unsigned OUTSIDE = 0xfffffff0u;
    const __amdgpu_buffer_rsrc_t r_panel = __builtin_amdgcn_make_buffer_rsrc(
        A + i0 + (int64_t)j0 * lda, 0, (int)(((int64_t)(nb - 1) * lda + nrows) * (int64_t)sizeof(T)), 0x00020000);
    auto panel_off = [&](int i, int d) -> unsigned {
        return (i < nrows && d < nb) ? (unsigned)(((int64_t)d * lda + i) * (int64_t)sizeof(T)) : OUTSIDE;
    };
    // the stripe into LDS: thread (i, dsub) takes columns dsub, dsub + TPR, ...; sixteen loads in flight
    if (!comm) {
        const int i = tid % RPW, dsub = tid / RPW;
        for (int d0 = 0; d0 < nb; d0 += 16 * TPR) {
            T v[16];
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const unsigned off = panel_off(i, d0 + dsub + q * TPR);
                if constexpr (sizeof(T) == 8) v[q] = __builtin_bit_cast(T, (u32x2)__builtin_amdgcn_raw_buffer_load_b64(r_panel, off, 0, 0));
                else v[q] = __builtin_bit_cast(T, (unsigned int)__builtin_amdgcn_raw_buffer_load_b32(r_panel, off, 0, 0));
            }
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const int d = d0 + dsub + q * TPR;
                if (d < nb) P[d * LS + i] = v[q];
            }
        }
    }
    if (tid == 0) s_abort = 0;
    __syncthreads();

    // computing thread (row ui, column group udsub); the TPR threads of a row are lanes of one wave, which reads
    // the row's multiplier in one instruction before any of them overwrites it
    const int ui = wave * RW + lane % RW, udsub = lane / RW;
    const int urow = i0 + ui;                               // global row
    const bool has_row = !comm && ui < nrows;
    // The communicator's own view of the stripe: rows lane, lane + 64, ... (RPW / 64 of them).  It finds the
    // candidates of a column itself, from what the column will hold once the pivot before is applied, with the
    // very operations the computing waves use (scaled() and eliminated() below), so that the magnitudes it
    // compares are those of the entries that get stored.
    constexpr int CR = RPW / 64;
    auto scaled = [](T x, int how, T rcp) -> T { return how == 1 ? x * rcp : (how == 2 ? x / rcp : x); };
    auto eliminated = [](T x, T l, T u) -> T {
        if constexpr (sizeof(T) == 8) return __builtin_fma(-l, u, x);
        else return __builtin_fmaf(-l, u, x);
    };
    // The communicator publishes, for the column that comes next, the stripe's candidate {magnitude, row, sequence
    // number}, the candidate's whole row and (workgroup 0) the row that will be row r, all as they will be once the
    // pivot at hand is applied: it works them out itself while the computing waves have not started on that pivot.
    // rowv / topv: this lane's two elements (columns lane and lane + 64) of those rows.
    Cand<T> lb{T(-1), NONE};
    T rowv[COOP_NB / 64], topv[COOP_NB / 64];
    auto publish = [&](int cn, bool header, bool rows) {    // for column cn: the header first, the rows when they are worked out
        if (G == 1) return;
        const int parn = cn & 1;
        const unsigned seqn = (unsigned)(j0 + cn) + 1u;
        auto item = [&](double v, unsigned w2, unsigned w3) -> u32x4 {
            const u32x2 w = __builtin_bit_cast(u32x2, v);
            u32x4 o;
            o[0] = w[0];
            o[1] = w[1];
            o[2] = w2;
            o[3] = w3;
            return o;
        };
        const __amdgpu_buffer_rsrc_t r_hdr = __builtin_amdgcn_make_buffer_rsrc(x_hdr + (size_t)parn * COOP_GMAX * 16, 0, G * 16, 0x00020000);
        const __amdgpu_buffer_rsrc_t r_mine = __builtin_amdgcn_make_buffer_rsrc(x_rows + ((size_t)g * 2 + parn) * COOP_NB * 16, 0,
                                                                                COOP_NB * 16, 0x00020000);
        const __amdgpu_buffer_rsrc_t r_top = __builtin_amdgcn_make_buffer_rsrc(x_top + (size_t)parn * COOP_NB * 16, 0, COOP_NB * 16,
                                                                               0x00020000);
        if (header && lane == 0) __builtin_amdgcn_raw_buffer_store_b128(item((double)lb.val, (unsigned)lb.row, seqn), r_hdr, g * 16, 0, THROUGH);
#pragma unroll
        for (int q = 0; q < COOP_NB / 64; ++q) {
            const int d = lane + 64 * q;
            if (rows && d < nb) {
                __builtin_amdgcn_raw_buffer_store_b128(item((double)rowv[q], seqn, 0u), r_mine, d * 16, 0, THROUGH);
                if (g == 0) __builtin_amdgcn_raw_buffer_store_b128(item((double)topv[q], seqn, 0u), r_top, d * 16, 0, THROUGH);
            }
        }
    };
    if (comm) {
        Cand<T> mine{T(-1), NONE};
#pragma unroll
        for (int k = 0; k < CR; ++k) {
            const int i = lane + 64 * k;
            if (i < nrows) mine = better(mine, Cand<T>{abs_of(P[i]), i0 + i});
        }
        lb = wave_best(mine);
        const int ib = lb.row == NONE ? -1 : lb.row - i0;
#pragma unroll
        for (int q = 0; q < COOP_NB / 64; ++q) {
            const int d = lane + 64 * q;
            rowv[q] = (ib >= 0 && d < nb) ? P[d * LS + ib] : T(0);
            topv[q] = d < nb ? P[d * LS] : T(0);
        }
        publish(0, true, true);
    }

    bool aborted = false;
    int c_reached = 0;                                      // first column without a decision, if the panel is given up
    for (int c = 0; c < nb; ++c) {
        const int r = j0 + c, par = c & 1;
        const unsigned seq = (unsigned)r + 1u;
        T *const s_U = s_Ub[par], *const s_top = s_topb[par];
        int p = r;
        int spins = 0;
        bool fail = false;
        bool released = false;                              // the communicator has passed barrier C already
        if (comm) {
            if (G > 1) {
                const __amdgpu_buffer_rsrc_t r_hdr = __builtin_amdgcn_make_buffer_rsrc(x_hdr + (size_t)par * COOP_GMAX * 16, 0,
                                                                                       G * 16, 0x00020000);
                // poll: lane l looks at the headers l, l + 64, l + 128, l + 192 (past G: outside the buffer).  The first
                // look is put off by the time a published item takes to become visible: a look that comes too early
                // costs a whole round trip more
                for (int w = 0; w < hdr_delay; ++w) __builtin_amdgcn_s_sleep(1);
                Cand<double> cb{-1.0, NONE};
                for (;;) {
                    u32x4 h[COOP_GMAX / 64];
#pragma unroll
                    for (int q = 0; q < COOP_GMAX / 64; ++q)
                        h[q] = (u32x4)__builtin_amdgcn_raw_buffer_load_b128(r_hdr, (lane + 64 * q) * 16, 0, THROUGH);
                    const unsigned fl = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(r_flag, 0, 0, THROUGH);
                    bool ok = true;
                    cb = Cand<double>{-1.0, NONE};
#pragma unroll
                    for (int q = 0; q < COOP_GMAX / 64; ++q) {
                        if (lane + 64 * q < G) {
                            ok = ok && (h[q][3] == seq);
                            u32x2 vv;
                            vv[0] = h[q][0];
                            vv[1] = h[q][1];
                            cb = better(cb, Cand<double>{__builtin_bit_cast(double, vv), (int)h[q][2]});
                        }
                    }
                    if (__builtin_amdgcn_ballot_w64(!ok) == 0ull) break;
                    if (++spins > spin_limit || __builtin_amdgcn_readfirstlane((int)fl) != 0) { fail = true; break; }
                    __builtin_amdgcn_s_sleep(1);
                }
                if (!fail) {
                    cb = wave_best(cb);
                    const int best_row = __builtin_amdgcn_readfirstlane(cb.row);
                    const bool nobody = best_row == NONE;   // no candidate anywhere (a column of NaNs): row r stays
                    p = nobody ? r : best_row;
                    const int gp = (p - j0) / RPW;
                    const __amdgpu_buffer_rsrc_t r_win = __builtin_amdgcn_make_buffer_rsrc(x_rows + ((size_t)gp * 2 + par) * COOP_NB * 16, 0,
                                                                                           COOP_NB * 16, 0x00020000);
                    const __amdgpu_buffer_rsrc_t r_top = __builtin_amdgcn_make_buffer_rsrc(x_top + (size_t)par * COOP_NB * 16, 0,
                                                                                           COOP_NB * 16, 0x00020000);
                    const __amdgpu_buffer_rsrc_t r_u = nobody ? r_top : r_win;
                    // the pivot's row as its owner published it with its header, and row r: read again until every
                    // item carries this column's sequence number
                    for (int w = 0; w < row_delay; ++w) __builtin_amdgcn_s_sleep(1);
                    for (;;) {
                        u32x4 uv[COOP_NB / 64], tv[COOP_NB / 64];
#pragma unroll
                        for (int q = 0; q < COOP_NB / 64; ++q) {
                            uv[q] = (u32x4)__builtin_amdgcn_raw_buffer_load_b128(r_u, (lane + 64 * q) * 16, 0, THROUGH);
                            tv[q] = (u32x4)__builtin_amdgcn_raw_buffer_load_b128(r_top, (lane + 64 * q) * 16, 0, THROUGH);
                        }
                        const unsigned fl = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(r_flag, 0, 0, THROUGH);
                        bool ok = true;
#pragma unroll
                        for (int q = 0; q < COOP_NB / 64; ++q)
                            if (lane + 64 * q < nb) ok = ok && uv[q][2] == seq && tv[q][2] == seq;
                        if (__builtin_amdgcn_ballot_w64(!ok) == 0ull) {
#pragma unroll
                            for (int q = 0; q < COOP_NB / 64; ++q) {
                                const int d = lane + 64 * q;
                                if (d < nb) {
                                    u32x2 ua, ta;
                                    ua[0] = uv[q][0];
                                    ua[1] = uv[q][1];
                                    ta[0] = tv[q][0];
                                    ta[1] = tv[q][1];
                                    s_U[d] = (T)__builtin_bit_cast(double, ua);
                                    s_top[d] = (T)__builtin_bit_cast(double, ta);
                                }
                            }
                            break;
                        }
                        if (++spins > spin_limit || __builtin_amdgcn_readfirstlane((int)fl) != 0) { fail = true; break; }
                        __builtin_amdgcn_s_sleep(1);
                    }
                }
            } else {
                // one workgroup: its own candidate is the pivot, the rows are in this wave's registers
                p = lb.row == NONE ? r : __builtin_amdgcn_readfirstlane(lb.row);
#pragma unroll
                for (int q = 0; q < COOP_NB / 64; ++q) {
                    const int d = lane + 64 * q;
                    if (d < nb) {
                        s_U[d] = lb.row == NONE ? topv[q] : rowv[q];
                        s_top[d] = topv[q];
                    }
                }
            }
        }
        __syncthreads();                                    // B: the stripe is up to date with column c - 1
        if (comm) {
            if (fail) {
                if (lane == 0) {
                    __builtin_amdgcn_raw_buffer_store_b32(1u, r_flag, 0, 0, THROUGH);
                    s_abort = 1;
                }
            } else {
                // what every computing thread needs of the pivot, worked out once: the column is scaled by the
                // pivot's reciprocal as LAPACK does (one division per column; |a| <= |pivot| still gives
                // |a * (1 / pivot)| <= 1 after rounding) unless the reciprocal would overflow
                __builtin_amdgcn_s_waitcnt(0xC07F);         // lgkmcnt(0): this wave's writes of s_U and s_top have landed
                // Everything the steps below need from LDS that does not depend on their results is asked for here,
                // in one batch with the pivot, and chosen from afterwards: written with a branch per case this wave
                // made eight LDS round trips in a row, and all other waves of all workgroups wait for it.
                const bool more = c + 1 < nb;               // there is a next column
                const int cn = more ? c + 1 : c, it = cn;   // row r + 1 is local row c + 1 of workgroup 0
                const T pivot = s_U[c];
                T xc[CR], x1[CR], pt[COOP_NB / 64], su[COOP_NB / 64], st[COOP_NB / 64];
#pragma unroll
                for (int k = 0; k < CR; ++k) {
                    xc[k] = P[c * LS + lane + 64 * k];
                    x1[k] = P[cn * LS + lane + 64 * k];
                }
                const T u1 = s_U[cn], t0 = s_top[c], t1 = s_top[cn], lt_raw = P[c * LS + it];
#pragma unroll
                for (int q = 0; q < COOP_NB / 64; ++q) {
                    const int d = lane + 64 * q, dq = d < nb ? d : nb - 1;
                    pt[q] = P[dq * LS + it];
                    su[q] = s_U[dq];
                    st[q] = s_top[dq];
                }
                // what every computing thread needs of the pivot, worked out once: the column is scaled by the
                // pivot's reciprocal as LAPACK does (one division per column; |a| <= |pivot| still gives
                // |a * (1 / pivot)| <= 1 after rounding) unless the reciprocal would overflow
                const bool nonzero = pivot != T(0), by_rcp = abs_of(pivot) >= RcpLimit<T>::tiny();
                const int how = !nonzero ? 0 : (by_rcp ? 1 : 2);
                const T rcp = by_rcp ? T(1) / pivot : pivot;
                if (lane == 0) {
                    s_p = p;
                    s_how = how;
                    s_rcp = rcp;
                    if (g == 0) {
                        ipiv[r] = p + 1;
                        if (!nonzero && *info == 0) *info = r + 1;
                    }
                }
                if (more) {
                    // What the stripe will hold once this pivot is applied (the row that takes the old row r is read
                    // from s_top, as the computing waves will do): the candidates of column c + 1 among the rows
                    // below row r
                    const bool exch = p != r;
                    Cand<T> mine{T(-1), NONE};
#pragma unroll
                    for (int k = 0; k < CR; ++k) {
                        const int i = lane + 64 * k, row = i0 + i;
                        const bool moved = exch && row == p;
                        const T y = eliminated(moved ? t1 : x1[k], scaled(moved ? t0 : xc[k], how, rcp), u1);
                        if (i < nrows && row > r) mine = better(mine, Cand<T>{abs_of(y), row});
                    }
                    lb = wave_best(mine);
                    publish(c + 1, true, false);
                    // the candidate's row and (workgroup 0) row r + 1, both as they will be
                    const int ib = lb.row == NONE ? -1 : __builtin_amdgcn_readfirstlane(lb.row) - i0;
                    const int ibs = ib >= 0 ? ib : 0;
                    T pr[COOP_NB / 64];
#pragma unroll
                    for (int q = 0; q < COOP_NB / 64; ++q) {
                        const int d = lane + 64 * q, dq = d < nb ? d : nb - 1;
                        pr[q] = P[dq * LS + ibs];
                    }
                    const T lb_raw = P[c * LS + ibs];
                    // that was the last look at the stripe: the computing waves may start on this pivot while the rows
                    // are worked out and published
                    __builtin_amdgcn_s_waitcnt(0xC07F);     // lgkmcnt(0): what was read from LDS is in registers
                    __syncthreads();                        // C
                    released = true;
                    const bool moved_b = exch && i0 + ibs == p, moved_t = exch && i0 + it == p;
                    const T l_b = scaled(moved_b ? t0 : lb_raw, how, rcp);
                    const T l_t = scaled(moved_t ? t0 : lt_raw, how, rcp);
#pragma unroll
                    for (int q = 0; q < COOP_NB / 64; ++q) {
                        const int d = lane + 64 * q;
                        const T xb = moved_b ? st[q] : pr[q], xt = moved_t ? st[q] : pt[q];
                        const T vb = d < c ? xb : (d == c ? l_b : eliminated(xb, l_b, su[q]));
                        const T vt = d < c ? xt : (d == c ? l_t : eliminated(xt, l_t, su[q]));
                        rowv[q] = (ib >= 0 && d < nb) ? vb : T(0);
                        topv[q] = (g == 0 && d < nb) ? vt : T(0);
                    }
                    publish(c + 1, false, true);
                }
            }
        }
        if (!released) __syncthreads();                     // C: pivot row and row r in LDS, what to do with them known
        if (s_abort) { aborted = true; c_reached = c; break; }
        if (comm) continue;
        // the computing waves apply the pivot: the two rows change places, the column is scaled, the columns on its
        // right are updated; the communicator is already exchanging the candidates of the next column
        p = s_p;
        const int how = s_how;
        const T rcp = s_rcp;                                // the reciprocal, or the pivot itself where that would overflow
        const bool exchange = p != r;
        if (exchange && tid < nb) {
            // row r (local row c of workgroup 0) becomes the pivot row; the old row r goes where the pivot was: its
            // part left of column c here, the rest as the update below passes over that row
            if (g == 0) P[tid * LS + c] = s_U[tid];
            const int ip = p - i0;
            if (ip >= 0 && ip < RPW && tid < c) P[tid * LS + ip] = s_top[tid];
        }
        if (has_row && urow > r) {
            const bool moved = exchange && urow == p;
            const T l = scaled(moved ? s_top[c] : P[c * LS + ui], how, rcp);
            __builtin_amdgcn_wave_barrier();                // every thread of the row has read before one writes
            if (udsub == 0) P[c * LS + ui] = l;
            const bool any_moved = __builtin_amdgcn_ballot_w64(moved) != 0ull;
            const int e_last = (nb - 1) * LS + ui;
            // one piece: CH columns of the row per thread (CH * TPR columns of the panel from dbase on), all their
            // reads issued before the first write and none of them under a branch (columns past the panel read its
            // last column again and are not written)
            auto piece = [&](auto ch_tag, int dbase) {
                constexpr int CH = decltype(ch_tag)::value;
                const int d0 = dbase + udsub, e0 = d0 * LS + ui;
                T x[CH], uu[CH];
#pragma unroll
                for (int q = 0; q < CH; ++q) {
                    const int e = e0 + q * (TPR * LS), dq = d0 + q * TPR;
                    x[q] = P[e < e_last ? e : e_last];
                    uu[q] = s_U[dq < nb ? dq : nb - 1];
                }
                if (any_moved) {
#pragma unroll
                    for (int q = 0; q < CH; ++q) {
                        const int dq = d0 + q * TPR;
                        const T tv = s_top[dq < nb ? dq : nb - 1];
                        x[q] = moved ? tv : x[q];
                    }
                }
#pragma unroll
                for (int q = 0; q < CH; ++q) {
                    const int d = d0 + q * TPR;
                    if (d < nb) P[d * LS + ui] = eliminated(x[q], l, uu[q]);
                }
            };
            // pieces of 16 columns per thread, the last one of 8 or 4 where that covers what is left, so that the
            // last trip does not pay for columns that are not there
            int dbase = c + 1;
            for (; nb - dbase > 8 * TPR; dbase += 16 * TPR) piece(std::integral_constant<int, 16>{}, dbase);
            if (nb - dbase > 4 * TPR) piece(std::integral_constant<int, 8>{}, dbase);
            else if (nb - dbase > 0) piece(std::integral_constant<int, 4>{}, dbase);
        }
    }
    __syncthreads();
    if (aborted) {
        // The panel stays as it was found.  The interchanges this panel has not decided are recorded as "none":
        // the kernels that follow on the stream apply ipiv as it stands, and it must name rows of the matrix.
        if (g == 0) {
            for (int cc = c_reached + tid; cc < nb; cc += NTC + 64) ipiv[j0 + cc] = j0 + cc + 1;
            if (tid == 0) *info = COOP_INFO_TIMEOUT;
        }
        return;
    }
    // the stripe back to memory
    if (!comm) {
        const int i = tid % RPW, dsub = tid / RPW;
        for (int d = dsub; d < nb; d += TPR) {
            const T v = P[d * LS + i];
            const unsigned off = panel_off(i, d);
            if constexpr (sizeof(T) == 8) __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, v), r_panel, off, 0, 0);
            else __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, v), r_panel, off, 0, 0);
        }
    }
}

// Row interchanges k = k0 .. k1 - 1 (row k with row ipiv[k] - 1, in that order) applied to columns
// [c0, c1) of A: 32 columns per workgroup of one wave, one per thread (twice the workgroups of 64 columns each, so
// that every compute unit has one: the accesses are scattered lines, and the more units ask the better), 32
// interchanges per batch.
constexpr int SWAP_G = 32, SWAP_NT = 64, SWAP_COLS = 32;   // a wave per workgroup (its lanes are the slots of a batch), SWAP_COLS columns
template <typename T>
__global__ void __launch_bounds__(SWAP_NT) laswp_kernel(T *A, int64_t lda, int c0, int c1, int k0, int k1, const int *ipiv) {
    __shared__ SwapLds<T, SWAP_G, SWAP_COLS> s_swap;
    const int tid = threadIdx.x, c = tid < SWAP_COLS ? c0 + blockIdx.x * SWAP_COLS + tid : c1;
    T *const col = c < c1 ? A + (int64_t)c * lda : nullptr;
    for (int k = k0; k < k1; k += SWAP_G)
        swap_batch<T, SWAP_G, SWAP_COLS>(s_swap, col, k, ipiv + k, -1, (k1 - k) < SWAP_G ? (k1 - k) : SWAP_G, tid);
}

__global__ void clear_int_kernel(int *p) { *p = 0; }

template <typename T> struct Lu {
    T *A;
    int64_t lda;
    int64_t m, n;
    int *ipiv, *info;
    void *stream;
    unsigned char *xch;     // exchange memory of the shared panels (COOP_BYTES), or nullptr: no panel of several workgroups
    int ncu;                // compute units of the device: most workgroups that can share a panel

    // The panel [j0, j0 + nb) by all the workgroups its rows need (getrf_coop_kernel), if they can be resident
    // together and the panel's offsets fit 32 bits; 1: not taken (the caller falls back to the recursive panel).
    int coop_panel(int64_t j0, int64_t nb) const {
        using C = CoopCfg<T>;
        if (!shared || nb > COOP_NB) return 1;
        const int64_t G = (m - j0 + C::RPW - 1) / C::RPW;
        if (G > 1 && (!xch || G > ncu || G > COOP_GMAX)) return 1;      // one workgroup waits for nobody and exchanges nothing
        if ((int64_t)COOP_NB * lda * (int64_t)sizeof(T) >= (int64_t)0x7fffffff) return 1;
        constexpr size_t LDS = (size_t)COOP_NB * (C::RPW + 1) * sizeof(T);
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(getrf_coop_kernel<T, C::RPW, C::TPR>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
        if (attr != hipSuccess) return (int)attr;
        hipLaunchKernelGGL((getrf_coop_kernel<T, C::RPW, C::TPR>), dim3((unsigned)G), dim3(C::RPW * C::TPR + 64), LDS, static_cast<hipStream_t>(stream),
                           A, lda, (int)m, (int)j0, (int)nb, ipiv, info, xch, t_lu_spin_limit, t_lu_hdr_delay, t_lu_row_delay);
        return (int)hipGetLastError();
    }

    int trsm(int64_t rows, int64_t cols, const T *L, T *B) const;
    int gemm(int64_t mm, int64_t nn, int64_t kk, const T *X, const T *Y, T *C) const;

    int swap_rows(int64_t c0, int64_t c1, int64_t k0, int64_t k1) const {
        if (c1 <= c0 || k1 <= k0) return 0;
        hipLaunchKernelGGL(laswp_kernel<T>, dim3((unsigned)((c1 - c0 + SWAP_COLS - 1) / SWAP_COLS)), dim3(SWAP_NT), 0,
                           static_cast<hipStream_t>(stream), A, lda, (int)c0, (int)c1, (int)k0, (int)k1, ipiv);
        return (int)hipGetLastError();
    }

    // columns [j0, j0 + w) below and including row j0, w <= min(m, n) - j0, inside the panel [c_lo, c_hi) of the
    // sweep: the leaves carry their interchanges through all of that panel's columns
    // Widest leaf for rows j0 .. m - 1: what keeps the leaf in the registers of one workgroup (64 elements per
    // thread); leaves taller than that at a single column go through memory at full width.
    static constexpr int MIN_W = 1;
    int64_t leaf_width(int64_t j0) const {
        const int64_t rows_per_thread = (m - j0 + LEAF_NT - 1) / LEAF_NT;
        for (int64_t wd = LEAF; wd >= MIN_W; wd /= 2)
            if (rows_per_thread * wd <= leaf_elems<T>((int)wd)) return wd;
        return LEAF;
    }
    template <int W> int leaf(int64_t j0, int64_t w, int64_t c_lo, int64_t c_hi, bool resident, int pre, int post) const {
        const hipStream_t st = static_cast<hipStream_t>(stream);
        if (resident)
            hipLaunchKernelGGL((getf2_kernel<T, leaf_elems<T>(W) / W, W, true>), dim3(1), dim3(LEAF_NT), 0, st, A, lda, (int)m, (int)j0,
                               (int)w, (int)c_lo, (int)c_hi, ipiv, info, pre, post);
        else
            hipLaunchKernelGGL((getf2_kernel<T, leaf_elems<T>(W) / W, W, false>), dim3(1), dim3(LEAF_NT), 0, st, A, lda, (int)m, (int)j0,
                               (int)w, (int)c_lo, (int)c_hi, ipiv, info, 0, 0);
        return (int)hipGetLastError();
    }
    bool resident_at(int64_t j0, int64_t lw) const { return ((m - j0 + LEAF_NT - 1) / LEAF_NT) * lw <= leaf_elems<T>((int)lw); }
    int any_leaf(int64_t j0, int64_t w, int64_t c_lo, int64_t c_hi, int pre, int post) const {
        const int64_t lw = leaf_width(j0);
        const bool resident = resident_at(j0, lw);
        switch (lw) {
            case 8: return leaf<8>(j0, w, c_lo, c_hi, resident, pre, post);
            case 4: return leaf<4>(j0, w, c_lo, c_hi, resident, pre, post);
            case 2: return leaf<2>(j0, w, c_lo, c_hi, resident, pre, post);
            default: return leaf<1>(j0, w, c_lo, c_hi, resident, pre, post);
        }
    }
    // Columns [j0, j0 + w) inside the enclosing panel [c_lo, c_hi): halved down to base panels of at most `base`
    // columns; a base panel is shared by all the workgroups its rows need where there is exchange memory and it is
    // not too tall, else halved further down to leaves of one workgroup, and its interchanges are then applied to
    // the other columns of the enclosing panel by laswp_kernel (a leaf carries its interchanges only through its
    // own base panel: carried through a wide panel they cost more than everything else).
    int64_t base;
    bool shared;            // base panels in LDS (getrf_coop_kernel) where they can be; false: leaves of one workgroup only
    int panel(int64_t j0, int64_t w, int64_t c_lo, int64_t c_hi) const {
        int rc;
        if (w <= base) {
            rc = coop_panel(j0, w);
            if (rc == 1) rc = leaf_panel(j0, w, j0, j0 + w);
            if (rc) return rc;
            if ((rc = swap_rows(c_lo, j0, j0, j0 + w))) return rc;
            return swap_rows(j0 + w, c_hi, j0, j0 + w);
        }
        const int64_t w1 = ((w / 2 + base - 1) / base) * base, w2 = w - w1, j1 = j0 + w1;
        if ((rc = panel(j0, w1, c_lo, c_hi))) return rc;
        if ((rc = trsm(w1, w2, A + j0 + j0 * lda, A + j0 + j1 * lda))) return rc;
        if (m > j1 && (rc = gemm(m - j1, w2, w1, A + j1 + j0 * lda, A + j0 + j1 * lda, A + j1 + j1 * lda))) return rc;
        return panel(j1, w2, c_lo, c_hi);
    }
    int leaf_panel(int64_t j0, int64_t w, int64_t c_lo, int64_t c_hi) const {
        int rc;
        const int64_t lw = leaf_width(j0);
        if (w <= lw) return any_leaf(j0, w, c_lo, c_hi, 0, 0);
        const int64_t w1 = ((w / 2 + lw - 1) / lw) * lw, w2 = w - w1, j1 = j0 + w1;
        // Two leaves side by side, both in registers: the left one leaves the block row of U for the right one
        // behind (post), the right one applies the left one's update as it loads (pre), and neither the solve nor
        // the product between them is launched.
        const int64_t lw2 = leaf_width(j1);
        if (lw > 1 && lw2 > 1 && w1 <= lw && w2 <= lw2 && resident_at(j0, lw) && resident_at(j1, lw2)) {
            if ((rc = any_leaf(j0, w1, c_lo, c_hi, 0, (int)w2))) return rc;
            return any_leaf(j1, w2, c_lo, c_hi, (int)w1, 0);
        }
        if ((rc = leaf_panel(j0, w1, c_lo, c_hi))) return rc;
        T *const A11 = A + j0 + j0 * lda, *const A12 = A + j0 + j1 * lda;
        T *const A21 = A + j1 + j0 * lda, *const A22 = A + j1 + j1 * lda;
        if ((rc = trsm(w1, w2, A11, A12))) return rc;
        if (m > j1 && (rc = gemm(m - j1, w2, w1, A21, A12, A22))) return rc;
        return leaf_panel(j1, w2, c_lo, c_hi);
    }

    int run() const {
        const int64_t steps = min64(m, n);
        // The whole matrix is one panel, halved down to base panels: the products between the halves are as deep as they
        // can be and interchanges are applied level by level to as few columns as possible (against a sweep over panels
        // of 128 columns: dgetrf_ws 16384 139 -> 127 ms, 32768 677 -> 521; dgetrf 16384 311 -> 296; no difference at
        // 8192).  A forced width W sweeps over panels of W columns, each halved the same way.
        const int64_t W = t_lu_panel > 0 ? t_lu_panel : max64(steps, 1);
        int rc;
        for (int64_t j = 0; j < steps; j += W) {
            const int64_t nb = min64(W, steps - j), j1 = j + nb;
            if ((rc = panel(j, nb, j, j1))) return rc;
            if ((rc = swap_rows(0, j, j, j1))) return rc;
            if (j1 < n) {
                if ((rc = swap_rows(j1, n, j, j1))) return rc;
                if ((rc = trsm(nb, n - j1, A + j + j * lda, A + j + j1 * lda))) return rc;
                if (j1 < m && (rc = gemm(m - j1, n - j1, nb, A + j1 + j * lda, A + j + j1 * lda, A + j1 + j1 * lda))) return rc;
            }
        }
        return 0;
    }
};

template <> int Lu<double>::trsm(int64_t rows, int64_t cols, const double *L, double *B) const {
    return xgemm_dtrsm('L', 'L', 'N', 'U', rows, cols, 1.0, L, lda, B, lda, stream);
}
template <> int Lu<float>::trsm(int64_t rows, int64_t cols, const float *L, float *B) const {
    return xgemm_strsm('L', 'L', 'N', 'U', rows, cols, 1.0f, L, lda, B, lda, stream);
}
template <> int Lu<double>::gemm(int64_t mm, int64_t nn, int64_t kk, const double *X, const double *Y, double *C) const {
    return xgemm_dgemm('N', 'N', mm, nn, kk, -1.0, X, lda, Y, lda, 1.0, C, lda, stream);
}
template <> int Lu<float>::gemm(int64_t mm, int64_t nn, int64_t kk, const float *X, const float *Y, float *C) const {
    return xgemm_sgemm('N', 'N', mm, nn, kk, -1.0f, X, lda, Y, lda, 1.0f, C, lda, stream);
}

// Per process and device: what orders the factorisations with shared panels, and the exchange buffer of those
// that bring none.
struct SharedPanels {
    static constexpr int MAX_DEV = 64;
    std::mutex mu;
    unsigned char *buf = nullptr;
    hipEvent_t done = nullptr;
    bool used = false, alloc_failed = false;
};
SharedPanels g_shared_panels[SharedPanels::MAX_DEV];

template <typename T>
int getrf_impl(int64_t m, int64_t n, T *A, int64_t lda, int *ipiv, int *info, void *work, size_t lwork, void *stream) {
    if (m < 0 || m > DIM_MAX) return -1;
    if (n < 0 || n > DIM_MAX) return -2;
    if (m > 0 && n > 0 && !A) return -3;
    if (lda < max64(1, m)) return -4;
    if (m > 0 && n > 0 && !ipiv) return -5;
    if (!info) return -6;
    if (work && (reinterpret_cast<uintptr_t>(work) & 15)) return -7;
    hipLaunchKernelGGL(clear_int_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream), info);
    int rc = (int)hipGetLastError();
    if (rc || m == 0 || n == 0) return rc;
    // Panels shared by several workgroups need exchange memory: the caller's, else one buffer per device that
    // the library allocates the first time it is needed (never while the stream is being captured: then, and if
    // the allocation fails, only panels of a single workgroup and the leaves are used).  Workgroups of a shared
    // panel wait for each other, and two factorisations whose panels cannot all be resident together could each
    // hold the compute units the other waits for; so every factorisation with shared panels on a device is
    // ordered behind the one before it, whichever thread and stream it comes from (an event recorded at the end
    // of each, waited for at the start of the next, both under a lock that is held while the kernels are
    // enqueued).  A captured call can take no part in that order: it is up to the caller there.
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if ((rc = (int)hipStreamIsCapturing(st, &capturing))) return rc;
    const bool captured = capturing != hipStreamCaptureStatusNone;
    const bool want_shared = t_lu_shared != 0;
    unsigned char *xch = (want_shared && work && lwork >= COOP_BYTES) ? static_cast<unsigned char *>(work) : nullptr;
    int dev = 0, ncu = 0;
    if ((rc = (int)hipGetDevice(&dev))) return rc;
    if ((rc = (int)hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev))) return rc;
    SharedPanels *sp = (want_shared && !captured && dev >= 0 && dev < SharedPanels::MAX_DEV) ? &g_shared_panels[dev] : nullptr;
    std::unique_lock<std::mutex> order;
    if (sp) {
        order = std::unique_lock<std::mutex>(sp->mu);
        if (!sp->done && hipEventCreateWithFlags(&sp->done, hipEventDisableTiming) != hipSuccess) sp->done = nullptr;
        if (!sp->done) {
            (void)hipGetLastError();
            order.unlock();
            sp = nullptr;
            if (!captured) xch = nullptr;             // without the order no shared panels outside a capture
        } else {
            if (!xch) {
                if (!sp->buf && !sp->alloc_failed && hipMalloc(reinterpret_cast<void **>(&sp->buf), COOP_BYTES) != hipSuccess) {
                    (void)hipGetLastError();
                    sp->buf = nullptr;
                    sp->alloc_failed = true;
                }
                xch = sp->buf;
            }
            if (xch && sp->used && (rc = (int)hipStreamWaitEvent(st, sp->done, 0))) return rc;
        }
    }
    if (xch) {
        hipLaunchKernelGGL(coop_clear_kernel, dim3(64), dim3(256), 0, st, reinterpret_cast<uint4 *>(xch));
        if ((rc = (int)hipGetLastError())) return rc;
    }
    const int64_t steps = min64(m, n), base_default = (want_shared || steps >= 4096) ? 128 : 64;
    const Lu<T> lu{A, lda, m, n, ipiv, info, stream, xch, ncu, t_lu_panel > 0 ? min64(t_lu_panel, base_default) : base_default, want_shared};
    rc = lu.run();
    if (sp && xch) {
        const int rec = (int)hipEventRecord(sp->done, st);
        sp->used = sp->used || rec == 0;
        if (!rc) rc = rec;
    }
    return rc;
}

}  // namespace

namespace xg {
void reset_lu_tuning() {
    t_lu_panel = -1;
    t_lu_spin_limit = 1 << 18;
    t_lu_shared = -1;
    t_lu_hdr_delay = LU_HDR_DELAY;
    t_lu_row_delay = LU_ROW_DELAY;
}
}  // namespace xg

extern "C" {

int xgemm_dgetrf(int64_t m, int64_t n, double *A, int64_t lda, int *ipiv, int *info, void *stream) {
    return getrf_impl<double>(m, n, A, lda, ipiv, info, nullptr, 0, stream);
}

int xgemm_sgetrf(int64_t m, int64_t n, float *A, int64_t lda, int *ipiv, int *info, void *stream) {
    return getrf_impl<float>(m, n, A, lda, ipiv, info, nullptr, 0, stream);
}

size_t xgemm_getrf_workspace_bytes(void) { return COOP_BYTES; }

int xgemm_dgetrf_ws(int64_t m, int64_t n, double *A, int64_t lda, int *ipiv, int *info, void *work, size_t lwork, void *stream) {
    return getrf_impl<double>(m, n, A, lda, ipiv, info, work, lwork, stream);
}

int xgemm_sgetrf_ws(int64_t m, int64_t n, float *A, int64_t lda, int *ipiv, int *info, void *work, size_t lwork, void *stream) {
    return getrf_impl<float>(m, n, A, lda, ipiv, info, work, lwork, stream);
}

int xgemm_force_getrf_poll_delay(int header_sleeps, int row_sleeps) {
    if (header_sleeps < 0 || row_sleeps < 0 || header_sleeps > 1024 || row_sleeps > 1024) return -1;
    t_lu_hdr_delay = header_sleeps;
    t_lu_row_delay = row_sleeps;
    return 0;
}

int xgemm_force_getrf_shared(int mode) {
    if (mode != -1 && mode != 0) return -1;
    t_lu_shared = mode;
    return 0;
}

int xgemm_force_getrf_spin_limit(int polls) {
    if (polls < 0) return -1;
    t_lu_spin_limit = polls;
    return 0;
}

int xgemm_force_getrf_panel(int64_t width) {
    if (width < -1 || width == 0 || width > DIM_MAX) return -1;
    t_lu_panel = width;
    return 0;
}

}  // extern "C"
