// xgemm_lu.hip -- LU factorisation with partial pivoting on the level-3 routines (the other
// LAPACK-level driver the paper names as resting on GEMM, Abstract and Sec. 1).
//
//     P A = L U,   A m x n,  L unit lower trapezoidal, U upper trapezoidal, both in place;
//     ipiv[j] (1-based) is the row that was interchanged with row j at step j.
//
// Organisation.  The matrix is swept right-looking in panels of PANEL columns.  A panel is
// factored recursively by halving its columns (left half; interchanges, triangular solve and
// product for the right half; right half; interchanges for the left half), so that all
// arithmetic of a panel except its leaves runs in the solve and product kernels.  A leaf of up
// to LEAF columns is factored by ONE workgroup (getf2_kernel): the search for the pivot is a
// reduction inside the workgroup, so nothing in the library ever waits for another workgroup,
// and a leaf costs one launch, not one per column.  After a panel its interchanges are applied
// to the columns on both sides of it (laswp_kernel), the block row of U comes from a triangular
// solve and the rest of the matrix is updated by one product of depth PANEL.
#include "../../include/xgemm.h"
#include "../../include/xgemm_tuning.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

inline int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }
inline int64_t min64(int64_t a, int64_t b) { return a < b ? a : b; }
constexpr int64_t DIM_MAX = 0x7fffffff;
constexpr int LEAF = 8;          // columns one workgroup factors by itself
constexpr int LEAF_NT = 1024;    // its threads
constexpr int LEAF_WAVES = LEAF_NT / 64;

thread_local int64_t t_lu_panel = -1;   // -1: by the order; W > 0: panels of W columns

template <typename T> __device__ __forceinline__ T abs_of(T x) { return x < T(0) ? -x : x; }

// Candidate for the pivot: the largest magnitude, and among equal magnitudes the smallest row.
template <typename T> struct Cand {
    T val;
    int row;
};
template <typename T> __device__ __forceinline__ Cand<T> better(Cand<T> a, Cand<T> b) {
    return (b.val > a.val || (b.val == a.val && b.row < a.row)) ? b : a;
}
template <typename T> __device__ __forceinline__ Cand<T> wave_best(Cand<T> c) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        Cand<T> o;
        o.val = __shfl_xor(c.val, d, 64);
        o.row = __shfl_xor(c.row, d, 64);
        c = better(c, o);
    }
    return c;
}

// Columns [j0, j0 + w) of A, rows j0 .. m - 1, w <= LEAF: Gaussian elimination with partial pivoting, one
// column at a time, by one workgroup; the leaf stays in memory (the caches of this CU), the rows are dealt to
// the threads.  Per column: the pivot is the first largest entry (reduction over the workgroup); the pivot row
// and row j0 + c change places within the leaf's columns; the column is divided by the pivot (a true division,
// so that no multiplier exceeds one); the columns to its right inside the leaf are updated, and the search for
// the next column's pivot rides on that pass.  A zero pivot is recorded in *info (first one only, 1-based
// column) and its column left as it is.  ipiv[j0 + c] receives the pivot's row + 1.
template <typename T>
__global__ void __launch_bounds__(LEAF_NT) getf2_kernel(T *A, int64_t lda, int m, int j0, int w, int *ipiv, int *info) {
    __shared__ T s_val[LEAF_WAVES];
    __shared__ int s_row[LEAF_WAVES];
    __shared__ int s_piv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    T *const P = A + (int64_t)j0 * lda;          // column j0 of the matrix
    Cand<T> mine{T(-1), 0x7fffffff};
    for (int i = j0 + tid; i < m; i += LEAF_NT) {
        const T v = abs_of(P[i]);
        if (v > mine.val) { mine.val = v; mine.row = i; }
    }
    for (int c = 0; c < w; ++c) {
        const int r = j0 + c;
        // the pivot of column c
        const Cand<T> wb = wave_best(mine);
        if (lane == 0) { s_val[wave] = wb.val; s_row[wave] = wb.row; }
        __syncthreads();
        if (wave == 0) {
            Cand<T> x{lane < LEAF_WAVES ? s_val[lane & (LEAF_WAVES - 1)] : T(-1), lane < LEAF_WAVES ? s_row[lane & (LEAF_WAVES - 1)] : 0x7fffffff};
            x = wave_best(x);
            if (lane == 0) {
                s_piv = x.row;
                ipiv[r] = x.row + 1;
                if (x.val == T(0) && *info == 0) *info = r + 1;
            }
        }
        __syncthreads();
        const int p = s_piv;
        T *const Pc = P + (int64_t)c * lda;
        const bool nonzero = Pc[p] != T(0);
        __syncthreads();                          // everybody has read the pivot before rows move
        if (tid < w && p != r && nonzero) {
            T *const q = P + (int64_t)tid * lda;
            const T x = q[r];
            q[r] = q[p];
            q[p] = x;
        }
        __syncthreads();
        const T pivot = Pc[r];
        T u[LEAF];
#pragma unroll
        for (int d = 1; d < LEAF; ++d) u[d] = (c + d < w) ? P[r + (int64_t)(c + d) * lda] : T(0);
        mine.val = T(-1);
        mine.row = 0x7fffffff;
        for (int i = r + 1 + tid; i < m; i += LEAF_NT) {
            T l = Pc[i];
            if (nonzero) {
                l = l / pivot;
                Pc[i] = l;
            }
#pragma unroll
            for (int d = 1; d < LEAF; ++d) {
                if (c + d < w) {
                    T *const q = P + i + (int64_t)(c + d) * lda;
                    const T x = *q - l * u[d];
                    *q = x;
                    if (d == 1) {
                        const T v = abs_of(x);
                        if (v > mine.val) { mine.val = v; mine.row = i; }
                    }
                }
            }
        }
        __syncthreads();                          // the updated columns are complete before the next search reads them
    }
}

// Row interchanges k = k0 .. k1 - 1 (row k with row ipiv[k] - 1, in that order) applied to columns
// [c0, c1) of A; one thread per column.
template <typename T>
__global__ void __launch_bounds__(256) laswp_kernel(T *A, int64_t lda, int c0, int c1, int k0, int k1, const int *ipiv) {
    const int col = c0 + blockIdx.x * 256 + threadIdx.x;
    if (col >= c1) return;
    T *const q = A + (int64_t)col * lda;
    for (int k = k0; k < k1; ++k) {
        const int p = ipiv[k] - 1;
        if (p != k) {
            const T x = q[k];
            q[k] = q[p];
            q[p] = x;
        }
    }
}

__global__ void clear_int_kernel(int *p) { *p = 0; }

template <typename T> struct Lu {
    T *A;
    int64_t lda;
    int64_t m, n;
    int *ipiv, *info;
    void *stream;

    int trsm(int64_t rows, int64_t cols, const T *L, T *B) const;
    int gemm(int64_t mm, int64_t nn, int64_t kk, const T *X, const T *Y, T *C) const;

    int swap_rows(int64_t c0, int64_t c1, int64_t k0, int64_t k1) const {
        if (c1 <= c0 || k1 <= k0) return 0;
        hipLaunchKernelGGL(laswp_kernel<T>, dim3((unsigned)((c1 - c0 + 255) / 256)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), A, lda, (int)c0, (int)c1, (int)k0, (int)k1, ipiv);
        return (int)hipGetLastError();
    }

    // columns [j0, j0 + w) below and including row j0, w <= min(m, n) - j0; interchanges stay inside those columns
    int panel(int64_t j0, int64_t w) const {
        if (w <= LEAF) {
            hipLaunchKernelGGL(getf2_kernel<T>, dim3(1), dim3(LEAF_NT), 0, static_cast<hipStream_t>(stream), A, lda, (int)m,
                               (int)j0, (int)w, ipiv, info);
            return (int)hipGetLastError();
        }
        const int64_t w1 = ((w / 2 + LEAF - 1) / LEAF) * LEAF, w2 = w - w1, j1 = j0 + w1;
        int rc;
        if ((rc = panel(j0, w1))) return rc;
        if ((rc = swap_rows(j1, j0 + w, j0, j1))) return rc;
        T *const A11 = A + j0 + j0 * lda, *const A12 = A + j0 + j1 * lda;
        T *const A21 = A + j1 + j0 * lda, *const A22 = A + j1 + j1 * lda;
        if ((rc = trsm(w1, w2, A11, A12))) return rc;
        if (m > j1 && (rc = gemm(m - j1, w2, w1, A21, A12, A22))) return rc;
        if ((rc = panel(j1, w2))) return rc;
        return swap_rows(j0, j1, j1, j0 + w);
    }

    int run() const {
        const int64_t steps = min64(m, n);
        const int64_t W = t_lu_panel > 0 ? t_lu_panel : (steps >= 4096 ? 128 : 64);
        int rc;
        for (int64_t j = 0; j < steps; j += W) {
            const int64_t nb = min64(W, steps - j), j1 = j + nb;
            if ((rc = panel(j, nb))) return rc;
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

template <typename T> int getrf_impl(int64_t m, int64_t n, T *A, int64_t lda, int *ipiv, int *info, void *stream) {
    if (m < 0 || m > DIM_MAX) return -1;
    if (n < 0 || n > DIM_MAX) return -2;
    if (m > 0 && n > 0 && !A) return -3;
    if (lda < max64(1, m)) return -4;
    if (m > 0 && n > 0 && !ipiv) return -5;
    if (!info) return -6;
    hipLaunchKernelGGL(clear_int_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream), info);
    const int rc = (int)hipGetLastError();
    if (rc || m == 0 || n == 0) return rc;
    const Lu<T> lu{A, lda, m, n, ipiv, info, stream};
    return lu.run();
}

}  // namespace

namespace xg {
void reset_lu_tuning() { t_lu_panel = -1; }
}  // namespace xg

extern "C" {

int xgemm_dgetrf(int64_t m, int64_t n, double *A, int64_t lda, int *ipiv, int *info, void *stream) {
    return getrf_impl<double>(m, n, A, lda, ipiv, info, stream);
}

int xgemm_sgetrf(int64_t m, int64_t n, float *A, int64_t lda, int *ipiv, int *info, void *stream) {
    return getrf_impl<float>(m, n, A, lda, ipiv, info, stream);
}

int xgemm_force_getrf_panel(int64_t width) {
    if (width < -1 || width == 0 || width > DIM_MAX) return -1;
    t_lu_panel = width;
    return 0;
}

}  // extern "C"
