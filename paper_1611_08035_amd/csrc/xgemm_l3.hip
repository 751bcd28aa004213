// xgemm_l3.hip -- level-3 routines on top of the GEMM entry points: the
// triangular solve with many right-hand sides.
//
// The solve is organised so that almost all of its arithmetic is GEMM: the
// triangular matrix is halved recursively, each half is solved in turn, and
// the coupling between the halves is one product with the off-diagonal block
// (depth = half the order, so the products are large).  Diagonal blocks of
// order <= NB are solved by substitution in a small kernel of their own.
#include "../../include/xgemm.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int NB = 64;        // order of the diagonal blocks solved by substitution
constexpr int LDE = NB + 2;   // LDS column stride of the block (keeps 16-byte alignment, spreads banks)

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
};

// One wave solves E x = b for 64 right-hand sides, one per lane, the unsolved
// part of x in registers.  E is brought to lower-triangular form in LDS (an
// upper-triangular E is reversed in both indices, and the right-hand sides with
// it), stored by columns with the reciprocals of the diagonal kept apart.
// Step c takes the pivot from register 0, stores it, and eliminates it from
// the rows below while shifting them down one register:
//   x_c = reg[0] / E_cc;   reg[i] = reg[i+1] - E(c+1+i, c) x_c,  i = 0..NB-2
// so the registers are indexed statically inside a loop over c that stays a
// loop.  Registers whose row lies beyond the block pick up whatever LDS holds
// past the column and are never used as pivots.  All lanes read the same
// element of E at the same time (LDS broadcast).
template <typename T> __global__ void __launch_bounds__(64) trsm_block_kernel(const BlockArgs<T> a) {
    __shared__ T e_cols[(NB + 1) * LDE];   // one spare column: reads below the last row stay inside the array
    __shared__ T d_inv[NB];
    const int t = threadIdx.x;
    const int nbk = a.nbk;
    const bool e_lower = (a.stored_lower != 0) != (a.etrans != 0);

    for (int i = t; i < (NB + 1) * LDE; i += 64) e_cols[i] = T(0);
    d_inv[t] = T(1);
    __syncthreads();
    // stored column s, stored row t: only the referenced triangle is read
    for (int s = 0; s < nbk; ++s) {
        const bool inside = t < nbk && (a.stored_lower ? t >= s : t <= s) && !(a.unit && t == s);
        if (inside) {
            const T v = a.A[t + (int64_t)s * a.lda];
            int r = a.etrans ? s : t, c = a.etrans ? t : s;
            if (!e_lower) { r = nbk - 1 - r; c = nbk - 1 - c; }
            if (r == c) d_inv[r] = T(1) / v;
            else e_cols[c * LDE + r] = v;
        }
    }
    __syncthreads();

    const int q = blockIdx.x * 64 + t;
    const bool active = q < a.nrhs;
    // lanes past the last right-hand side work on a copy of the last one and store nothing;
    // positions past the block's order re-read its first element and are replaced by zero:
    // every load is in bounds and none is conditional
    const int qq = active ? q : a.nrhs - 1;
    const int64_t xs = a.left ? 1 : a.ldb;                       // stride inside a right-hand side
    T *const xp = a.B + (a.left ? (int64_t)qq * a.ldb : (int64_t)qq);
    const int64_t first = e_lower ? 0 : (int64_t)(nbk - 1) * xs, step = e_lower ? xs : -xs;
    T x[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const T v = xp[first + (i < nbk ? i : 0) * step];
        x[i] = i < nbk ? v : T(0);
    }
#pragma unroll 1
    for (int c = 0; c < nbk; ++c) {
        const T xc = x[0] * d_inv[c];
        if (active) xp[first + c * step] = xc;
        const T *const col = e_cols + c * LDE + c + 1;
#pragma unroll
        for (int i = 0; i + 1 < NB; ++i) x[i] = x[i + 1] - col[i] * xc;
        x[NB - 1] = T(0);
    }
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

template <typename T> struct Solve {
    bool left, stored_lower, trans, unit;
    const T *A;
    int64_t lda;
    T *B;
    int64_t ldb, m, n;
    void *stream;

    // E = op(T) for side L, op(T)^T for side R; the solve runs first-block-first when E is lower
    bool etrans() const { return trans != !left; }
    bool forward() const { return stored_lower != etrans(); }

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
        hipLaunchKernelGGL(trsm_block_kernel<T>, dim3((unsigned)((a.nrhs + 63) / 64)), dim3(64), 0,
                           static_cast<hipStream_t>(stream), a);
        return (int)hipGetLastError();
    }

    // rows/columns [off, off + dim) of the triangular matrix against the matching part of B
    int run(int64_t off, int64_t dim) const {
        if (dim <= NB) return block(off, dim);
        const int64_t n1 = ((dim / 2 + NB - 1) / NB) * NB, n2 = dim - n1;
        // the off-diagonal block of the stored triangle: T21 (n2 x n1) or T12 (n1 x n2)
        const T *blk = stored_lower ? A + (off + n1) + off * lda : A + off + (off + n1) * lda;
        const char tc = trans ? 'T' : 'N';
        int rc;
        if (forward()) {
            if ((rc = run(off, n1))) return rc;
            if (left)   // B2 -= op(T)21 X1
                rc = real_gemm<T>(tc, 'N', n2, n, n1, T(-1), blk, lda, B + off, ldb, T(1), B + off + n1, ldb, stream);
            else        // B2 -= X1 op(T)12
                rc = real_gemm<T>('N', tc, m, n2, n1, T(-1), B + off * ldb, ldb, blk, lda, T(1), B + (off + n1) * ldb,
                                  ldb, stream);
            if (rc) return rc;
            return run(off + n1, n2);
        }
        if ((rc = run(off + n1, n2))) return rc;
        if (left)       // B1 -= op(T)12 X2
            rc = real_gemm<T>(tc, 'N', n1, n, n2, T(-1), blk, lda, B + off + n1, ldb, T(1), B + off, ldb, stream);
        else            // B1 -= X2 op(T)21
            rc = real_gemm<T>('N', tc, m, n1, n2, T(-1), B + (off + n1) * ldb, ldb, blk, lda, T(1), B + off * ldb, ldb,
                              stream);
        if (rc) return rc;
        return run(off, n1);
    }
};

template <typename T>
int trsm_impl(char side, char uplo, char transa, char diag, int64_t m, int64_t n, T alpha, const T *A, int64_t lda,
              T *B, int64_t ldb, void *stream) {
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
    if (m == 0 || n == 0) return 0;
    if (alpha != T(1)) {
        const dim3 grid((unsigned)((m + 255) / 256), (unsigned)(n < 1024 ? n : 1024));
        hipLaunchKernelGGL(scale_b_kernel<T>, grid, dim3(256), 0, static_cast<hipStream_t>(stream), B, ldb, (int)m, (int)n,
                           alpha);
        const int rc = (int)hipGetLastError();
        if (rc || alpha == T(0)) return rc;
    }
    Solve<T> s{left, lower, is_t(transa), unit, A, lda, B, ldb, m, n, stream};
    return s.run(0, left ? m : n);
}

}  // namespace

extern "C" {

int xgemm_dtrsm(char side, char uplo, char transa, char diag, int64_t m, int64_t n, double alpha, const double *A,
                int64_t lda, double *B, int64_t ldb, void *stream) {
    return trsm_impl<double>(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb, stream);
}

int xgemm_strsm(char side, char uplo, char transa, char diag, int64_t m, int64_t n, float alpha, const float *A,
                int64_t lda, float *B, int64_t ldb, void *stream) {
    return trsm_impl<float>(side, uplo, transa, diag, m, n, alpha, A, lda, B, ldb, stream);
}

}  // extern "C"
