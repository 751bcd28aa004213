/*
 * ref_gemm.c -- CPU oracle for the real and split-plane complex GEMM.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct
 * definition that the GPU library is compared against.  It shares no code with
 * the GPU path and must never be called from it.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg use it.
 *
 * What it computes.  The paper (Sec. 2.1) writes the micro-kernel as
 *     C += A B = sum_{p=0}^{k_c-1} a_p b_p^T          (a_p column of A, b_p^T row of B)
 * and the loop nest of Fig. 1 sums those micro-kernel calls over all blocks.
 * Blocking, packing and unit updates (Sec. 2.2) only change the ORDER of the
 * k-sum, never its exact-arithmetic value, so the oracle is that value written
 * out as a triple loop with the k-sum taken in natural order p = 0..k-1:
 *
 *     C[i + j*ldc] <- alpha * sum_p opA(i,p) * opB(p,j) + beta * C[i + j*ldc]
 *     opA(i,p) = A[i + p*lda]  (trans 'N')   or  A[p + i*lda]  (trans 'T'/'C')
 *     opB(p,j) = B[p + j*ldb]  (trans 'N')   or  B[j + p*ldb]  (trans 'T'/'C')
 *
 * The scalars alpha/beta, transposes, leading dimensions and argument checks
 * are not in the paper (its kernel is C += AB); they follow the column-major
 * BLAS convention:
 *   - beta == 0  : C is write-only (NaN/Inf in C do not propagate);
 *   - alpha == 0 or k == 0 : A and B are not read;
 *   - m == 0 or n == 0 : nothing is touched;
 *   - rows m..ldc-1 of every column of C are never touched;
 *   - return 0, or -(1-based index) of the first illegal argument in the order
 *     transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc.
 *
 * Two accumulation modes:
 *   *_work : accumulator in the working precision, separate multiply and add
 *            (build with -ffp-contract=off).  In place on C.  This is the timed
 *            CPU baseline and the reference for the bit-exact integer cases.
 *   *_ext  : accumulator one level wider (float -> double, double -> x87
 *            long double with a 64-bit significand).  Writes the reference
 *            value and the magnitude G = |alpha| |opA| |opB| + |beta| |C_in|
 *            to separate dense m x n arrays of the wide type, so the
 *            comparison  |C_gpu - C_ref| <= 4 k u G  sees a reference whose own
 *            error is far below the bound.
 *
 * Loop order is j (column of C), p, i: each C(i,j) still receives its products
 * in the order p = 0,1,..,k-1; the i loop is innermost only so that the
 * column-major operands are walked with unit stride.  OpenMP splits the j
 * loop; every thread owns whole columns of C, so results do not depend on the
 * thread count.
 */
#include <stddef.h>
#include <stdlib.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef long long i64;

static int is_n(char t) { return t == 'N' || t == 'n'; }
static int is_t(char t) { return t == 'T' || t == 't' || t == 'C' || t == 'c'; }
static int is_conj(char t) { return t == 'C' || t == 'c'; }
static i64 max64(i64 a, i64 b) { return a > b ? a : b; }

/* Argument check shared by all entry points (BLAS xerbla numbering). */
static int check_args(char ta, char tb, i64 m, i64 n, i64 k,
                      const void *A, i64 lda, const void *B, i64 ldb,
                      const void *C, i64 ldc, int ab_needed)
{
    if (!is_n(ta) && !is_t(ta)) return -1;
    if (!is_n(tb) && !is_t(tb)) return -2;
    if (m < 0) return -3;
    if (n < 0) return -4;
    if (k < 0) return -5;
    i64 rows_a = is_n(ta) ? m : k;
    i64 rows_b = is_n(tb) ? k : n;
    if (ab_needed && m > 0 && n > 0 && k > 0 && A == NULL) return -7;
    if (lda < max64(1, rows_a)) return -8;
    if (ab_needed && m > 0 && n > 0 && k > 0 && B == NULL) return -9;
    if (ldb < max64(1, rows_b)) return -10;
    if (m > 0 && n > 0 && C == NULL) return -12;
    if (ldc < max64(1, m)) return -13;
    return 0;
}

int ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void ref_set_num_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

#define OPA(i, p) (an ? A[(i) + (p) * lda] : A[(p) + (i) * lda])
#define OPB(p, j) (bn ? B[(p) + (j) * ldb] : B[(j) + (p) * ldb])

/* ------------------------------------------------------------------ */
/* Working-precision GEMM, in place.                                    */
/* ------------------------------------------------------------------ */
#define DEFINE_REF_GEMM_WORK(NAME, T)                                          \
int NAME(char ta, char tb, i64 m, i64 n, i64 k, T alpha, const T *A, i64 lda,  \
         const T *B, i64 ldb, T beta, T *C, i64 ldc)                           \
{                                                                              \
    int need_ab = (alpha != (T)0);                                             \
    int info = check_args(ta, tb, m, n, k, A, lda, B, ldb, C, ldc, need_ab);   \
    if (info) return info;                                                     \
    if (m == 0 || n == 0) return 0;                                            \
    if ((alpha == (T)0 || k == 0) && beta == (T)1) return 0;                   \
    const int an = is_n(ta), bn = is_n(tb);                                    \
    int failed = 0;                                                            \
    _Pragma("omp parallel")                                                    \
    {                                                                          \
        T *acc = (T *)malloc((size_t)m * sizeof(T));                           \
        if (!acc) {                                                            \
            _Pragma("omp atomic write")                                        \
            failed = 1;                                                        \
        }                                                                      \
        _Pragma("omp for schedule(static)")                                    \
        for (i64 j = 0; j < n; ++j) {                                          \
            if (!acc) continue;                                                \
            T *Cj = C + j * ldc;                                               \
            if (alpha == (T)0 || k == 0) {                                     \
                for (i64 i = 0; i < m; ++i)                                    \
                    Cj[i] = (beta == (T)0) ? (T)0 : beta * Cj[i];              \
                continue;                                                      \
            }                                                                  \
            for (i64 i = 0; i < m; ++i) acc[i] = (T)0;                         \
            for (i64 p = 0; p < k; ++p) {                                      \
                const T b = OPB(p, j);                                         \
                for (i64 i = 0; i < m; ++i) {                                  \
                    T prod = OPA(i, p) * b;                                    \
                    acc[i] = acc[i] + prod;                                    \
                }                                                              \
            }                                                                  \
            for (i64 i = 0; i < m; ++i) {                                      \
                T t = alpha * acc[i];                                          \
                if (beta == (T)0) Cj[i] = t;                                   \
                else { T bc = beta * Cj[i]; Cj[i] = t + bc; }                  \
            }                                                                  \
        }                                                                      \
        free(acc);                                                             \
    }                                                                          \
    return failed ? 1000 : 0;                                                  \
}

DEFINE_REF_GEMM_WORK(ref_dgemm_work, double)
DEFINE_REF_GEMM_WORK(ref_sgemm_work, float)

/* ------------------------------------------------------------------ */
/* Extended-precision GEMM: reference value and magnitude G.            */
/* Cref and G are dense m x n, column-major, leading dimension m.       */
/* C_in is read only when beta != 0.                                    */
/* ------------------------------------------------------------------ */
#define DEFINE_REF_GEMM_EXT(NAME, T, W, WABS)                                  \
int NAME(char ta, char tb, i64 m, i64 n, i64 k, T alpha, const T *A, i64 lda,  \
         const T *B, i64 ldb, T beta, const T *C, i64 ldc, W *Cref, W *G)      \
{                                                                              \
    int need_ab = (alpha != (T)0);                                             \
    int info = check_args(ta, tb, m, n, k, A, lda, B, ldb, C, ldc, need_ab);   \
    if (info) return info;                                                     \
    if (m == 0 || n == 0) return 0;                                            \
    const int an = is_n(ta), bn = is_n(tb);                                    \
    const int use_ab = (alpha != (T)0 && k > 0);                               \
    int failed = 0;                                                            \
    _Pragma("omp parallel")                                                    \
    {                                                                          \
        W *acc = (W *)malloc((size_t)m * sizeof(W));                           \
        W *mag = (W *)malloc((size_t)m * sizeof(W));                           \
        if (!acc || !mag) {                                                    \
            _Pragma("omp atomic write")                                        \
            failed = 1;                                                        \
        }                                                                      \
        _Pragma("omp for schedule(static)")                                    \
        for (i64 j = 0; j < n; ++j) {                                          \
            if (!acc || !mag) continue;                                        \
            for (i64 i = 0; i < m; ++i) { acc[i] = 0; mag[i] = 0; }            \
            if (use_ab) {                                                      \
                for (i64 p = 0; p < k; ++p) {                                  \
                    const W b = (W)OPB(p, j);                                  \
                    for (i64 i = 0; i < m; ++i) {                              \
                        W prod = (W)OPA(i, p) * b;                             \
                        acc[i] += prod;                                        \
                        mag[i] += WABS(prod);                                  \
                    }                                                          \
                }                                                              \
            }                                                                  \
            for (i64 i = 0; i < m; ++i) {                                      \
                W r = (W)alpha * acc[i];                                       \
                W g = WABS((W)alpha) * mag[i];                                 \
                if (beta != (T)0) {                                            \
                    W c = (W)C[i + j * ldc];                                   \
                    r += (W)beta * c;                                          \
                    g += WABS((W)beta) * WABS(c);                              \
                }                                                              \
                Cref[i + j * m] = r;                                           \
                G[i + j * m] = g;                                              \
            }                                                                  \
        }                                                                      \
        free(acc);                                                             \
        free(mag);                                                             \
    }                                                                          \
    return failed ? 1000 : 0;                                                  \
}

DEFINE_REF_GEMM_EXT(ref_dgemm_ext, double, long double, fabsl)
DEFINE_REF_GEMM_EXT(ref_sgemm_ext, float, double, fabs)

/* ------------------------------------------------------------------ */
/* Single entries in extended precision: for parity at sizes where the  */
/* full triple loop is too slow.  Entry s is C(I[s], J[s]).             */
/* ------------------------------------------------------------------ */
#define DEFINE_REF_GEMM_SAMPLES(NAME, T, W, WABS)                              \
int NAME(char ta, char tb, i64 m, i64 n, i64 k, T alpha, const T *A, i64 lda,  \
         const T *B, i64 ldb, T beta, const T *C, i64 ldc, i64 ns,             \
         const i64 *I, const i64 *J, W *cref, W *g)                            \
{                                                                              \
    int need_ab = (alpha != (T)0);                                             \
    int info = check_args(ta, tb, m, n, k, A, lda, B, ldb, C, ldc, need_ab);   \
    if (info) return info;                                                     \
    const int an = is_n(ta), bn = is_n(tb);                                    \
    const int use_ab = (alpha != (T)0 && k > 0);                               \
    int bad = 0;                                                               \
    _Pragma("omp parallel for schedule(static)")                               \
    for (i64 s = 0; s < ns; ++s) {                                             \
        const i64 i = I[s], j = J[s];                                          \
        if (i < 0 || i >= m || j < 0 || j >= n) {                              \
            _Pragma("omp atomic write")                                        \
            bad = 1;                                                           \
            continue;                                                          \
        }                                                                      \
        W acc = 0, mag = 0;                                                    \
        if (use_ab) {                                                          \
            for (i64 p = 0; p < k; ++p) {                                      \
                W prod = (W)OPA(i, p) * (W)OPB(p, j);                          \
                acc += prod;                                                   \
                mag += WABS(prod);                                             \
            }                                                                  \
        }                                                                      \
        W r = (W)alpha * acc;                                                  \
        W gg = WABS((W)alpha) * mag;                                           \
        if (beta != (T)0) {                                                    \
            W c = (W)C[i + j * ldc];                                           \
            r += (W)beta * c;                                                  \
            gg += WABS((W)beta) * WABS(c);                                     \
        }                                                                      \
        cref[s] = r;                                                           \
        g[s] = gg;                                                             \
    }                                                                          \
    return bad ? -14 : 0;                                                      \
}

DEFINE_REF_GEMM_SAMPLES(ref_dgemm_samples, double, long double, fabsl)
DEFINE_REF_GEMM_SAMPLES(ref_sgemm_samples, float, double, fabs)


/* ------------------------------------------------------------------ */
/* Symmetric rank-k update on one triangle (level-3 BLAS on top of the  */
/* GEMM kernel, paper Abstract and Sec. 1):                             */
/*   C := alpha * op(A) * op(A)^T + beta * C,  op(A) is n x k,          */
/*   op(A)(i,p) = A[i + p*lda] (trans 'N') or A[p + i*lda] ('T'/'C').   */
/* Only entries with i >= j (uplo 'L') or i <= j ('U') are read and     */
/* written.  Same scalar rules as GEMM.  Errors: uplo 1, trans 2, n 3,  */
/* k 4, alpha 5, A 6, lda 7, beta 8, C 9, ldc 10.                       */
/* ------------------------------------------------------------------ */
static int check_args_syrk(char uplo, char t, i64 n, i64 k, const void *A, i64 lda, const void *C, i64 ldc,
                           int a_needed)
{
    if (uplo != 'L' && uplo != 'l' && uplo != 'U' && uplo != 'u') return -1;
    if (!is_n(t) && !is_t(t)) return -2;
    if (n < 0) return -3;
    if (k < 0) return -4;
    if (a_needed && n > 0 && k > 0 && A == NULL) return -6;
    if (lda < max64(1, is_n(t) ? n : k)) return -7;
    if (n > 0 && C == NULL) return -9;
    if (ldc < max64(1, n)) return -10;
    return 0;
}

#define OPS(i, p) (an ? A[(i) + (p) * lda] : A[(p) + (i) * lda])

#define DEFINE_REF_SYRK_WORK(NAME, T)                                          \
int NAME(char uplo, char t, i64 n, i64 k, T alpha, const T *A, i64 lda,        \
         T beta, T *C, i64 ldc)                                                \
{                                                                              \
    int info = check_args_syrk(uplo, t, n, k, A, lda, C, ldc, alpha != (T)0);  \
    if (info) return info;                                                     \
    if (n == 0) return 0;                                                      \
    if ((alpha == (T)0 || k == 0) && beta == (T)1) return 0;                   \
    const int an = is_n(t), lower = (uplo == 'L' || uplo == 'l');              \
    _Pragma("omp parallel for schedule(dynamic, 8)")                           \
    for (i64 j = 0; j < n; ++j) {                                              \
        const i64 i0 = lower ? j : 0, i1 = lower ? n : j + 1;                  \
        for (i64 i = i0; i < i1; ++i) {                                        \
            T acc = (T)0;                                                      \
            if (alpha != (T)0)                                                 \
                for (i64 p = 0; p < k; ++p) {                                  \
                    T prod = OPS(i, p) * OPS(j, p);                            \
                    acc = acc + prod;                                          \
                }                                                              \
            T r = alpha * acc;                                                 \
            if (alpha == (T)0 || k == 0) r = (T)0;                             \
            if (beta == (T)0) C[i + j * ldc] = r;                              \
            else { T bc = beta * C[i + j * ldc]; C[i + j * ldc] = r + bc; }    \
        }                                                                      \
    }                                                                          \
    return 0;                                                                  \
}

DEFINE_REF_SYRK_WORK(ref_dsyrk_work, double)
DEFINE_REF_SYRK_WORK(ref_ssyrk_work, float)

/* Extended precision: Cref and G are dense n x n (ld = n); entries outside the
 * triangle are set to 0 and carry no meaning. */
#define DEFINE_REF_SYRK_EXT(NAME, T, W, WABS)                                  \
int NAME(char uplo, char t, i64 n, i64 k, T alpha, const T *A, i64 lda,        \
         T beta, const T *C, i64 ldc, W *Cref, W *G)                           \
{                                                                              \
    int info = check_args_syrk(uplo, t, n, k, A, lda, C, ldc, alpha != (T)0);  \
    if (info) return info;                                                     \
    const int an = is_n(t), lower = (uplo == 'L' || uplo == 'l');              \
    const int use_a = (alpha != (T)0 && k > 0);                                \
    _Pragma("omp parallel for schedule(dynamic, 8)")                           \
    for (i64 j = 0; j < n; ++j) {                                              \
        for (i64 i = 0; i < n; ++i) { Cref[i + j * n] = 0; G[i + j * n] = 0; } \
        const i64 i0 = lower ? j : 0, i1 = lower ? n : j + 1;                  \
        for (i64 i = i0; i < i1; ++i) {                                        \
            W acc = 0, mag = 0;                                                \
            if (use_a)                                                         \
                for (i64 p = 0; p < k; ++p) {                                  \
                    W prod = (W)OPS(i, p) * (W)OPS(j, p);                      \
                    acc += prod;                                               \
                    mag += WABS(prod);                                         \
                }                                                              \
            W r = (W)alpha * acc, g = WABS((W)alpha) * mag;                    \
            if (beta != (T)0) {                                                \
                W c = (W)C[i + j * ldc];                                       \
                r += (W)beta * c;                                              \
                g += WABS((W)beta) * WABS(c);                                  \
            }                                                                  \
            Cref[i + j * n] = r;                                               \
            G[i + j * n] = g;                                                  \
        }                                                                      \
    }                                                                          \
    return 0;                                                                  \
}

DEFINE_REF_SYRK_EXT(ref_dsyrk_ext, double, long double, fabsl)
DEFINE_REF_SYRK_EXT(ref_ssyrk_ext, float, double, fabs)


/* ------------------------------------------------------------------ */
/* Triangular solve with many right-hand sides (level-3 BLAS on top of  */
/* the GEMM kernel, paper Abstract and Sec. 1):                         */
/*   side 'L':  op(T) X = alpha B,   T is m x m                         */
/*   side 'R':  X op(T) = alpha B,   T is n x n                         */
/* B (m x n) is overwritten by X.  Only the `uplo` triangle of the      */
/* stored T is read; diag 'U' takes a unit diagonal and does not read   */
/* the stored one.  alpha == 0 gives X = 0 without reading T or B.      */
/* Plain substitution, one right-hand side at a time: with E = op(T)    */
/* (side L) or op(T)^T (side R), row r of the solve is                  */
/*   x_r = (alpha b_r - sum_{c before r} E(r,c) x_c) / E(r,r).          */
/* Errors: side 1, uplo 2, trans 3, diag 4, m 5, n 6, alpha 7, A 8,     */
/* lda 9, B 10, ldb 11.                                                 */
/* ------------------------------------------------------------------ */
static int check_args_trsm(char side, char uplo, char t, char diag, i64 m, i64 n, int a_needed, const void *A,
                           i64 lda, const void *B, i64 ldb)
{
    const int left = (side == 'L' || side == 'l'), right = (side == 'R' || side == 'r');
    if (!left && !right) return -1;
    if (uplo != 'L' && uplo != 'l' && uplo != 'U' && uplo != 'u') return -2;
    if (!is_n(t) && !is_t(t)) return -3;
    if (diag != 'U' && diag != 'u' && diag != 'N' && diag != 'n') return -4;
    if (m < 0) return -5;
    if (n < 0) return -6;
    if (a_needed && m > 0 && n > 0 && A == NULL) return -8;
    if (lda < max64(1, left ? m : n)) return -9;
    if (m > 0 && n > 0 && B == NULL) return -10;
    if (ldb < max64(1, m)) return -11;
    return 0;
}

/* E(r,c) for the solve "E x = rhs": element (r,c) of op(T) for side L, of op(T)^T for side R */
#define TRI_E(r, c) (etrans ? A[(c) + (r) * lda] : A[(r) + (c) * lda])

#define DEFINE_REF_TRSM_WORK(NAME, T)                                          \
int NAME(char side, char uplo, char t, char diag, i64 m, i64 n, T alpha,       \
         const T *A, i64 lda, T *B, i64 ldb)                                   \
{                                                                              \
    int info = check_args_trsm(side, uplo, t, diag, m, n, alpha != (T)0, A, lda, B, ldb); \
    if (info) return info;                                                     \
    if (m == 0 || n == 0) return 0;                                            \
    const int left = (side == 'L' || side == 'l');                             \
    if (alpha == (T)0) {                                                       \
        for (i64 j = 0; j < n; ++j) for (i64 i = 0; i < m; ++i) B[i + j * ldb] = (T)0; \
        return 0;                                                              \
    }                                                                          \
    const int etrans = (is_t(t) ? 1 : 0) ^ (left ? 0 : 1);                     \
    const int lower = ((uplo == 'L' || uplo == 'l') ? 1 : 0) ^ etrans;         \
    const int unit = (diag == 'U' || diag == 'u');                             \
    const i64 dim = left ? m : n, nrhs = left ? n : m;                         \
    const i64 xs = left ? 1 : ldb, rs = left ? ldb : 1; /* strides inside / between right-hand sides */ \
    _Pragma("omp parallel for schedule(static)")                               \
    for (i64 q = 0; q < nrhs; ++q) {                                           \
        T *x = B + q * rs;                                                     \
        for (i64 step = 0; step < dim; ++step) {                               \
            const i64 r = lower ? step : dim - 1 - step;                       \
            T acc = alpha * x[r * xs];                                         \
            for (i64 s2 = 0; s2 < step; ++s2) {                                \
                const i64 c = lower ? s2 : dim - 1 - s2;                       \
                T prod = TRI_E(r, c) * x[c * xs];                              \
                acc = acc - prod;                                              \
            }                                                                  \
            x[r * xs] = unit ? acc : acc / TRI_E(r, r);                        \
        }                                                                      \
    }                                                                          \
    return 0;                                                                  \
}

DEFINE_REF_TRSM_WORK(ref_dtrsm_work, double)
DEFINE_REF_TRSM_WORK(ref_strsm_work, float)

/* Residual of a candidate solution X (m x n, leading dimension ldx) in extended
 * precision:  R = alpha B0 - op(T) X  (side L)  or  alpha B0 - X op(T)  (side R),
 * G = |alpha||B0| + |op(T)||X|  (resp. |X||op(T)|); R and G dense m x n, ld = m.
 * B0 is the right-hand side before the solve. */
#define DEFINE_REF_TRSM_RESID(NAME, T, W, WABS)                                \
int NAME(char side, char uplo, char t, char diag, i64 m, i64 n, T alpha,       \
         const T *A, i64 lda, const T *B0, i64 ldb, const T *X, i64 ldx,       \
         W *R, W *G)                                                           \
{                                                                              \
    int info = check_args_trsm(side, uplo, t, diag, m, n, 1, A, lda, B0, ldb); \
    if (info) return info;                                                     \
    if (m > 0 && n > 0 && X == NULL) return -12;                               \
    if (ldx < max64(1, m)) return -13;                                         \
    const int left = (side == 'L' || side == 'l');                             \
    const int etrans = (is_t(t) ? 1 : 0) ^ (left ? 0 : 1);                     \
    const int lower = ((uplo == 'L' || uplo == 'l') ? 1 : 0) ^ etrans;         \
    const int unit = (diag == 'U' || diag == 'u');                             \
    const i64 dim = left ? m : n;                                              \
    _Pragma("omp parallel for schedule(static)")                               \
    for (i64 j = 0; j < n; ++j)                                                \
        for (i64 i = 0; i < m; ++i) {                                          \
            /* the solve's row index r and right-hand side: (i, column j) or (j, row i) */ \
            const i64 r = left ? i : j;                                        \
            W acc = (W)alpha * (W)B0[i + j * ldb];                             \
            W mag = WABS(acc);                                                 \
            const i64 c0 = lower ? 0 : r, c1 = lower ? r + 1 : dim;            \
            for (i64 c = c0; c < c1; ++c) {                                    \
                W e = (c == r && unit) ? (W)1 : (W)TRI_E(r, c);                \
                W x = left ? (W)X[c + j * ldx] : (W)X[i + c * ldx];            \
                acc -= e * x;                                                  \
                mag += WABS(e * x);                                            \
            }                                                                  \
            R[i + j * m] = acc;                                                \
            G[i + j * m] = mag;                                                \
        }                                                                      \
    return 0;                                                                  \
}

DEFINE_REF_TRSM_RESID(ref_dtrsm_resid, double, long double, fabsl)
DEFINE_REF_TRSM_RESID(ref_strsm_resid, float, double, fabs)


/* The same residual at sampled entries only: R[s], G[s] for element (I[s], J[s]). */
#define DEFINE_REF_TRSM_RESID_SAMPLES(NAME, T, W, WABS)                        \
int NAME(char side, char uplo, char t, char diag, i64 m, i64 n, T alpha,       \
         const T *A, i64 lda, const T *B0, i64 ldb, const T *X, i64 ldx,       \
         i64 ns, const i64 *I, const i64 *J, W *R, W *G)                       \
{                                                                              \
    int info = check_args_trsm(side, uplo, t, diag, m, n, 1, A, lda, B0, ldb); \
    if (info) return info;                                                     \
    if (m > 0 && n > 0 && X == NULL) return -12;                               \
    if (ldx < max64(1, m)) return -13;                                         \
    for (i64 s = 0; s < ns; ++s)                                               \
        if (I[s] < 0 || I[s] >= m || J[s] < 0 || J[s] >= n) return -15;        \
    const int left = (side == 'L' || side == 'l');                             \
    const int etrans = (is_t(t) ? 1 : 0) ^ (left ? 0 : 1);                     \
    const int lower = ((uplo == 'L' || uplo == 'l') ? 1 : 0) ^ etrans;         \
    const int unit = (diag == 'U' || diag == 'u');                             \
    const i64 dim = left ? m : n;                                              \
    _Pragma("omp parallel for schedule(static)")                               \
    for (i64 s = 0; s < ns; ++s) {                                             \
        const i64 i = I[s], j = J[s];                                          \
        const i64 r = left ? i : j;                                            \
        W acc = (W)alpha * (W)B0[i + j * ldb];                                 \
        W mag = WABS(acc);                                                     \
        const i64 c0 = lower ? 0 : r, c1 = lower ? r + 1 : dim;                \
        for (i64 c = c0; c < c1; ++c) {                                        \
            W e = (c == r && unit) ? (W)1 : (W)TRI_E(r, c);                    \
            W x = left ? (W)X[c + j * ldx] : (W)X[i + c * ldx];                \
            acc -= e * x;                                                      \
            mag += WABS(e * x);                                                \
        }                                                                      \
        R[s] = acc;                                                            \
        G[s] = mag;                                                            \
    }                                                                          \
    return 0;                                                                  \
}

DEFINE_REF_TRSM_RESID_SAMPLES(ref_dtrsm_resid_samples, double, long double, fabsl)
DEFINE_REF_TRSM_RESID_SAMPLES(ref_strsm_resid_samples, float, double, fabs)


/* ------------------------------------------------------------------ */
/* Triangular matrix product (level-3 BLAS on top of the GEMM kernel):  */
/*   side 'L':  B := alpha op(T) B,   T is m x m                        */
/*   side 'R':  B := alpha B op(T),   T is n x n                        */
/* Same conventions as the triangular solve (only the `uplo` triangle   */
/* of T is read, diag 'U' implies ones; alpha == 0 gives B = 0 without  */
/* reading T or B).  Argument numbering as for the solve.  The result   */
/* is the definition: each element is the sum over the triangle in      */
/* increasing index order, times alpha.                                 */
/* ------------------------------------------------------------------ */
#define DEFINE_REF_TRMM(NAME, T, W, WABS)                                      \
/* Out (m x n, ld = m) = alpha op(T) B (or B op(T)) in precision W; G = |alpha| |op(T)| |B| */ \
int NAME(char side, char uplo, char t, char diag, i64 m, i64 n, T alpha,       \
         const T *A, i64 lda, const T *B, i64 ldb, W *Out, W *G)               \
{                                                                              \
    int info = check_args_trsm(side, uplo, t, diag, m, n, alpha != (T)0, A, lda, B, ldb); \
    if (info) return info;                                                     \
    const int left = (side == 'L' || side == 'l');                             \
    const int etrans = (is_t(t) ? 1 : 0) ^ (left ? 0 : 1);                     \
    const int lower = ((uplo == 'L' || uplo == 'l') ? 1 : 0) ^ etrans;         \
    const int unit = (diag == 'U' || diag == 'u');                             \
    const i64 dim = left ? m : n;                                              \
    _Pragma("omp parallel for schedule(static)")                               \
    for (i64 j = 0; j < n; ++j)                                                \
        for (i64 i = 0; i < m; ++i) {                                          \
            /* with E = op(T) (side L) or op(T)^T (side R): out = sum_c E(r, c) x_c */ \
            const i64 r = left ? i : j;                                        \
            W acc = 0, mag = 0;                                                \
            if (alpha != (T)0) {                                               \
                const i64 c0 = lower ? 0 : r, c1 = lower ? r + 1 : dim;        \
                for (i64 c = c0; c < c1; ++c) {                                \
                    W e = (c == r && unit) ? (W)1 : (W)TRI_E(r, c);            \
                    W x = left ? (W)B[c + j * ldb] : (W)B[i + c * ldb];        \
                    W prod = e * x;                                            \
                    acc = acc + prod;                                          \
                    mag += WABS(prod);                                         \
                }                                                              \
            }                                                                  \
            Out[i + j * m] = (alpha == (T)0) ? (W)0 : (W)alpha * acc;          \
            G[i + j * m] = WABS((W)alpha) * mag;                               \
        }                                                                      \
    return 0;                                                                  \
}

DEFINE_REF_TRMM(ref_dtrmm_ext, double, long double, fabsl)
DEFINE_REF_TRMM(ref_strmm_ext, float, double, fabs)
/* working precision (W = T): the bit-exact reference for integer data */
DEFINE_REF_TRMM(ref_dtrmm_wp, double, double, fabs)
DEFINE_REF_TRMM(ref_strmm_wp, float, float, fabsf)


/* ------------------------------------------------------------------ */
/* Cholesky factorisation (a LAPACK-level driver on top of the level-3  */
/* routines; the paper's motivation for a fast GEMM, Sec. 1):           */
/*   uplo 'L':  A = L L^T,  L lower triangular, overwrites the lower    */
/*   uplo 'U':  A = U^T U,  U upper triangular, overwrites the upper    */
/* triangle of the symmetric positive definite A; the other triangle is */
/* neither read nor written.  Column by column in the natural order:    */
/*   l_jj = sqrt(a_jj - sum_{p<j} l_jp^2),                              */
/*   l_ij = (a_ij - sum_{p<j} l_ip l_jp) / l_jj   (i > j).              */
/* Returns 0, -i for an illegal argument (uplo 1, n 2, A 3, lda 4), or  */
/* j > 0 if the leading minor of order j is not positive definite (the  */
/* factorisation stops there, as in LAPACK).                            */
/* ------------------------------------------------------------------ */
#define CH(i, j) (A[lower ? (i) + (j) * lda : (j) + (i) * lda])   /* element (i,j), i >= j, of L = U^T */

#define DEFINE_REF_POTRF(NAME, T, SQRT)                                        \
int NAME(char uplo, i64 n, T *A, i64 lda)                                      \
{                                                                              \
    const int lower = (uplo == 'L' || uplo == 'l');                            \
    if (!lower && uplo != 'U' && uplo != 'u') return -1;                       \
    if (n < 0) return -2;                                                      \
    if (n > 0 && A == NULL) return -3;                                         \
    if (lda < max64(1, n)) return -4;                                          \
    for (i64 j = 0; j < n; ++j) {                                              \
        T d = CH(j, j);                                                        \
        for (i64 p = 0; p < j; ++p) { T sq = CH(j, p) * CH(j, p); d = d - sq; }\
        if (!(d > (T)0)) return (int)(j + 1);                                  \
        d = SQRT(d);                                                           \
        CH(j, j) = d;                                                          \
        _Pragma("omp parallel for schedule(static) if (n - j > 256)")          \
        for (i64 i = j + 1; i < n; ++i) {                                      \
            T acc = CH(i, j);                                                  \
            for (i64 p = 0; p < j; ++p) { T prod = CH(i, p) * CH(j, p); acc = acc - prod; } \
            CH(i, j) = acc / d;                                                \
        }                                                                      \
    }                                                                          \
    return 0;                                                                  \
}

DEFINE_REF_POTRF(ref_dpotrf, double, sqrt)
DEFINE_REF_POTRF(ref_spotrf, float, sqrtf)

/* Residual of a candidate factor F against the original A0, on the `uplo`
 * triangle, in extended precision: R = A0 - L L^T, G = |L| |L|^T with L the
 * lower-triangular factor (F itself, or F^T for uplo 'U').  Either dense n x n
 * (ns < 0; entries outside the triangle are zero) or at ns sampled entries
 * (I[s], J[s]) of the triangle. */
#define FCH(i, j) (F[lower ? (i) + (j) * ldf : (j) + (i) * ldf])

#define DEFINE_REF_POTRF_RESID(NAME, T, W, WABS)                               \
int NAME(char uplo, i64 n, const T *A0, i64 lda, const T *F, i64 ldf,          \
         i64 ns, const i64 *I, const i64 *J, W *R, W *G)                       \
{                                                                              \
    const int lower = (uplo == 'L' || uplo == 'l');                            \
    if (!lower && uplo != 'U' && uplo != 'u') return -1;                       \
    if (n < 0) return -2;                                                      \
    if (n > 0 && A0 == NULL) return -3;                                        \
    if (lda < max64(1, n)) return -4;                                          \
    if (n > 0 && F == NULL) return -5;                                         \
    if (ldf < max64(1, n)) return -6;                                          \
    const i64 cnt = ns < 0 ? n * n : ns;                                       \
    for (i64 s = 0; s < (ns < 0 ? 0 : ns); ++s) {                              \
        if (I[s] < 0 || I[s] >= n || J[s] < 0 || J[s] >= n) return -8;         \
        if (lower ? I[s] < J[s] : I[s] > J[s]) return -8;                      \
    }                                                                          \
    _Pragma("omp parallel for schedule(dynamic, 64)")                          \
    for (i64 s = 0; s < cnt; ++s) {                                            \
        const i64 i = ns < 0 ? s % n : I[s], j = ns < 0 ? s / n : J[s];        \
        if (lower ? i < j : i > j) { R[s] = 0; G[s] = 0; continue; }           \
        const i64 hi = i > j ? i : j, lo = i > j ? j : i;   /* (L L^T)(hi, lo) = sum_{p <= lo} */ \
        W acc = (W)A0[i + j * lda], mag = 0;                                   \
        for (i64 p = 0; p <= lo; ++p) {                                        \
            W prod = (W)FCH(hi, p) * (W)FCH(lo, p);                            \
            acc -= prod;                                                       \
            mag += WABS(prod);                                                 \
        }                                                                      \
        R[s] = acc;                                                            \
        G[s] = mag;                                                            \
    }                                                                          \
    return 0;                                                                  \
}

DEFINE_REF_POTRF_RESID(ref_dpotrf_resid, double, long double, fabsl)
DEFINE_REF_POTRF_RESID(ref_spotrf_resid, float, double, fabs)


/* ------------------------------------------------------------------ */
/* The two remaining real level-3 routines on top of the GEMM kernel.   */
/*                                                                      */
/* Symmetric rank-2k update on one triangle:                            */
/*   C := alpha op(A) op(B)^T + alpha op(B) op(A)^T + beta C,           */
/*   op(X) n x k:  X(i,p) (trans 'N') or X(p,i) ('T'/'C').              */
/* Errors: uplo 1, trans 2, n 3, k 4, alpha 5, A 6, lda 7, B 8, ldb 9,  */
/* beta 10, C 11, ldc 12.  Out / G dense n x n (ld n), zero outside the  */
/* triangle; G = |alpha| (|op(A)||op(B)|^T + |op(B)||op(A)|^T) + |beta||C|. */
/*                                                                      */
/* Symmetric matrix product:                                            */
/*   side 'L':  C := alpha A B + beta C,  A m x m symmetric             */
/*   side 'R':  C := alpha B A + beta C,  A n x n symmetric             */
/* A is given by its `uplo` triangle; the other triangle is not read.   */
/* Errors: side 1, uplo 2, m 3, n 4, alpha 5, A 6, lda 7, B 8, ldb 9,   */
/* beta 10, C 11, ldc 12.  Out / G dense m x n (ld m).                  */
/* Sums run in increasing index order.                                  */
/* ------------------------------------------------------------------ */
#define OPX(X, ldx, i, p) (an ? X[(i) + (p) * (ldx)] : X[(p) + (i) * (ldx)])

#define DEFINE_REF_SYR2K(NAME, T, W, WABS)                                     \
int NAME(char uplo, char t, i64 n, i64 k, T alpha, const T *A, i64 lda,        \
         const T *B, i64 ldb, T beta, const T *C, i64 ldc, W *Out, W *G)       \
{                                                                              \
    const int lower = (uplo == 'L' || uplo == 'l');                            \
    if (!lower && uplo != 'U' && uplo != 'u') return -1;                       \
    if (!is_n(t) && !is_t(t)) return -2;                                       \
    if (n < 0) return -3;                                                      \
    if (k < 0) return -4;                                                      \
    const int an = is_n(t);                                                    \
    const int use_ab = (alpha != (T)0 && k > 0 && n > 0);                      \
    if (use_ab && A == NULL) return -6;                                        \
    if (lda < max64(1, an ? n : k)) return -7;                                 \
    if (use_ab && B == NULL) return -8;                                        \
    if (ldb < max64(1, an ? n : k)) return -9;                                 \
    if (n > 0 && C == NULL) return -11;                                        \
    if (ldc < max64(1, n)) return -12;                                         \
    _Pragma("omp parallel for schedule(dynamic, 8)")                           \
    for (i64 j = 0; j < n; ++j)                                                \
        for (i64 i = 0; i < n; ++i) {                                          \
            W acc = 0, mag = 0;                                                \
            if ((lower ? i >= j : i <= j)) {                                   \
                if (use_ab)                                                    \
                    for (i64 p = 0; p < k; ++p) {                              \
                        W p1 = (W)OPX(A, lda, i, p) * (W)OPX(B, ldb, j, p);    \
                        W p2 = (W)OPX(B, ldb, i, p) * (W)OPX(A, lda, j, p);    \
                        acc += p1; acc += p2;                                  \
                        mag += WABS(p1) + WABS(p2);                            \
                    }                                                          \
                acc = (W)alpha * acc;                                          \
                mag = WABS((W)alpha) * mag;                                    \
                if (beta != (T)0) {                                            \
                    W c = (W)C[i + j * ldc];                                   \
                    acc += (W)beta * c;                                        \
                    mag += WABS((W)beta) * WABS(c);                            \
                }                                                              \
            }                                                                  \
            Out[i + j * n] = acc;                                              \
            G[i + j * n] = mag;                                                \
        }                                                                      \
    return 0;                                                                  \
}

DEFINE_REF_SYR2K(ref_dsyr2k_ext, double, long double, fabsl)
DEFINE_REF_SYR2K(ref_ssyr2k_ext, float, double, fabs)
DEFINE_REF_SYR2K(ref_dsyr2k_wp, double, double, fabs)
DEFINE_REF_SYR2K(ref_ssyr2k_wp, float, float, fabsf)

/* element (r, c) of the symmetric A from its stored triangle */
#define SYM(r, c) ((lower ? (r) >= (c) : (r) <= (c)) ? A[(r) + (c) * lda] : A[(c) + (r) * lda])

#define DEFINE_REF_SYMM(NAME, T, W, WABS)                                      \
int NAME(char side, char uplo, i64 m, i64 n, T alpha, const T *A, i64 lda,     \
         const T *B, i64 ldb, T beta, const T *C, i64 ldc, W *Out, W *G)       \
{                                                                              \
    const int left = (side == 'L' || side == 'l');                             \
    const int lower = (uplo == 'L' || uplo == 'l');                            \
    if (!left && side != 'R' && side != 'r') return -1;                        \
    if (!lower && uplo != 'U' && uplo != 'u') return -2;                       \
    if (m < 0) return -3;                                                      \
    if (n < 0) return -4;                                                      \
    const int use_ab = (alpha != (T)0 && m > 0 && n > 0);                      \
    if (use_ab && A == NULL) return -6;                                        \
    if (lda < max64(1, left ? m : n)) return -7;                               \
    if (use_ab && B == NULL) return -8;                                        \
    if (ldb < max64(1, m)) return -9;                                          \
    if (m > 0 && n > 0 && C == NULL) return -11;                               \
    if (ldc < max64(1, m)) return -12;                                         \
    const i64 dim = left ? m : n;                                              \
    _Pragma("omp parallel for schedule(static)")                               \
    for (i64 j = 0; j < n; ++j)                                                \
        for (i64 i = 0; i < m; ++i) {                                          \
            W acc = 0, mag = 0;                                                \
            if (use_ab)                                                        \
                for (i64 c = 0; c < dim; ++c) {                                \
                    W prod = left ? (W)SYM(i, c) * (W)B[c + j * ldb]           \
                                  : (W)B[i + c * ldb] * (W)SYM(c, j);          \
                    acc += prod;                                               \
                    mag += WABS(prod);                                         \
                }                                                              \
            acc = (W)alpha * acc;                                              \
            mag = WABS((W)alpha) * mag;                                        \
            if (beta != (T)0) {                                                \
                W c = (W)C[i + j * ldc];                                       \
                acc += (W)beta * c;                                            \
                mag += WABS((W)beta) * WABS(c);                                \
            }                                                                  \
            Out[i + j * m] = acc;                                              \
            G[i + j * m] = mag;                                                \
        }                                                                      \
    return 0;                                                                  \
}

DEFINE_REF_SYMM(ref_dsymm_ext, double, long double, fabsl)
DEFINE_REF_SYMM(ref_ssymm_ext, float, double, fabs)
DEFINE_REF_SYMM(ref_dsymm_wp, double, double, fabs)
DEFINE_REF_SYMM(ref_ssymm_wp, float, float, fabsf)

/* ------------------------------------------------------------------ */
/* Complex GEMM on split real/imaginary planes.                         */
/*   C := alpha * op(A) * op(B) + beta * C,  op in {N, T, C(onj-transp)}*/
/* Each complex product is written out as 4 real multiplies and 2       */
/* add/subs; the k-sum of each component runs in natural order.         */
/* alpha = (alpha[0], alpha[1]), beta likewise.                         */
/* beta == (0,0): C is write-only.  alpha == (0,0) or k == 0: A, B not  */
/* read.  Argument numbering for errors: transa 1, transb 2, m 3, n 4,  */
/* k 5, alpha 6, Ar 7, Ai 8, lda 9, Br 10, Bi 11, ldb 12, beta 13,      */
/* Cr 14, Ci 15, ldc 16.                                                */
/* ------------------------------------------------------------------ */
static int check_args_z(char ta, char tb, i64 m, i64 n, i64 k, const double *alpha,
                        const void *Ar, const void *Ai, i64 lda,
                        const void *Br, const void *Bi, i64 ldb, const double *beta,
                        const void *Cr, const void *Ci, i64 ldc)
{
    if (!is_n(ta) && !is_t(ta)) return -1;
    if (!is_n(tb) && !is_t(tb)) return -2;
    if (m < 0) return -3;
    if (n < 0) return -4;
    if (k < 0) return -5;
    if (!alpha) return -6;
    if (!beta) return -13;
    int need_ab = (alpha[0] != 0.0 || alpha[1] != 0.0) && m > 0 && n > 0 && k > 0;
    i64 rows_a = is_n(ta) ? m : k;
    i64 rows_b = is_n(tb) ? k : n;
    if (need_ab && !Ar) return -7;
    if (need_ab && !Ai) return -8;
    if (lda < max64(1, rows_a)) return -9;
    if (need_ab && !Br) return -10;
    if (need_ab && !Bi) return -11;
    if (ldb < max64(1, rows_b)) return -12;
    if (m > 0 && n > 0 && !Cr) return -14;
    if (m > 0 && n > 0 && !Ci) return -15;
    if (ldc < max64(1, m)) return -16;
    return 0;
}

#define ZA(P, i, p) (an ? P[(i) + (p) * lda] : P[(p) + (i) * lda])
#define ZB(P, p, j) (bn ? P[(p) + (j) * ldb] : P[(j) + (p) * ldb])

/* Extended precision; outputs dense m x n (ld = m) long double planes:
 * reference (Rr, Ri) and magnitudes (Gr, Gi) where
 *   Gr = |al_r| (|Ar||Br| + |Ai||Bi|) + |al_i| (|Ar||Bi| + |Ai||Br|) + |be_r||Cr| + |be_i||Ci|
 * i.e. the sum of the absolute values of every real product that enters Cr,
 * and Gi likewise with the roles of the real and imaginary parts exchanged. */
int ref_zgemm_split_ext(char ta, char tb, i64 m, i64 n, i64 k, const double *alpha,
                        const double *Ar, const double *Ai, i64 lda,
                        const double *Br, const double *Bi, i64 ldb, const double *beta,
                        const double *Cr, const double *Ci, i64 ldc,
                        long double *Rr, long double *Ri, long double *Gr, long double *Gi)
{
    int info = check_args_z(ta, tb, m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb, beta, Cr, Ci, ldc);
    if (info) return info;
    if (m == 0 || n == 0) return 0;
    const int an = is_n(ta), bn = is_n(tb);
    const long double sa = is_conj(ta) ? -1.0L : 1.0L; /* sign of Im(op(A)) */
    const long double sb = is_conj(tb) ? -1.0L : 1.0L;
    const long double alr = alpha[0], ali = alpha[1], ber = beta[0], bei = beta[1];
    const int use_ab = (alr != 0 || ali != 0) && k > 0;
    const int use_c = (ber != 0 || bei != 0);
#pragma omp parallel for schedule(static)
    for (i64 j = 0; j < n; ++j) {
        for (i64 i = 0; i < m; ++i) {
            long double pr = 0, pi = 0, mr = 0, mi = 0;
            if (use_ab) {
                for (i64 p = 0; p < k; ++p) {
                    long double ar = ZA(Ar, i, p), ai = sa * ZA(Ai, i, p);
                    long double br = ZB(Br, p, j), bi = sb * ZB(Bi, p, j);
                    long double rr = ar * br, ii = ai * bi, ri = ar * bi, ir = ai * br;
                    pr += rr - ii;
                    pi += ri + ir;
                    mr += fabsl(rr) + fabsl(ii);
                    mi += fabsl(ri) + fabsl(ir);
                }
            }
            long double cr = alr * pr - ali * pi;
            long double ci = alr * pi + ali * pr;
            long double gr = fabsl(alr) * mr + fabsl(ali) * mi;
            long double gi = fabsl(alr) * mi + fabsl(ali) * mr;
            if (use_c) {
                long double c0 = Cr[i + j * ldc], c1 = Ci[i + j * ldc];
                cr += ber * c0 - bei * c1;
                ci += ber * c1 + bei * c0;
                gr += fabsl(ber) * fabsl(c0) + fabsl(bei) * fabsl(c1);
                gi += fabsl(ber) * fabsl(c1) + fabsl(bei) * fabsl(c0);
            }
            Rr[i + j * m] = cr; Ri[i + j * m] = ci;
            Gr[i + j * m] = gr; Gi[i + j * m] = gi;
        }
    }
    return 0;
}

/* Single entries (I[s], J[s]) of the complex reference, extended precision. */
int ref_zgemm_split_samples(char ta, char tb, i64 m, i64 n, i64 k, const double *alpha,
                            const double *Ar, const double *Ai, i64 lda,
                            const double *Br, const double *Bi, i64 ldb, const double *beta,
                            const double *Cr, const double *Ci, i64 ldc, i64 ns, const i64 *I, const i64 *J,
                            long double *rr_out, long double *ri_out, long double *gr_out, long double *gi_out)
{
    int info = check_args_z(ta, tb, m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb, beta, Cr, Ci, ldc);
    if (info) return info;
    const int an = is_n(ta), bn = is_n(tb);
    const long double sa = is_conj(ta) ? -1.0L : 1.0L;
    const long double sb = is_conj(tb) ? -1.0L : 1.0L;
    const long double alr = alpha[0], ali = alpha[1], ber = beta[0], bei = beta[1];
    const int use_ab = (alr != 0 || ali != 0) && k > 0;
    const int use_c = (ber != 0 || bei != 0);
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (i64 s = 0; s < ns; ++s) {
        const i64 i = I[s], j = J[s];
        if (i < 0 || i >= m || j < 0 || j >= n) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        long double pr = 0, pi = 0, mr = 0, mi = 0;
        if (use_ab) {
            for (i64 p = 0; p < k; ++p) {
                long double ar = ZA(Ar, i, p), ai = sa * ZA(Ai, i, p);
                long double br = ZB(Br, p, j), bi = sb * ZB(Bi, p, j);
                long double rr = ar * br, ii = ai * bi, ri = ar * bi, ir = ai * br;
                pr += rr - ii;
                pi += ri + ir;
                mr += fabsl(rr) + fabsl(ii);
                mi += fabsl(ri) + fabsl(ir);
            }
        }
        long double cr = alr * pr - ali * pi;
        long double ci = alr * pi + ali * pr;
        long double gr = fabsl(alr) * mr + fabsl(ali) * mi;
        long double gi = fabsl(alr) * mi + fabsl(ali) * mr;
        if (use_c) {
            long double c0 = Cr[i + j * ldc], c1 = Ci[i + j * ldc];
            cr += ber * c0 - bei * c1;
            ci += ber * c1 + bei * c0;
            gr += fabsl(ber) * fabsl(c0) + fabsl(bei) * fabsl(c1);
            gi += fabsl(ber) * fabsl(c1) + fabsl(bei) * fabsl(c0);
        }
        rr_out[s] = cr; ri_out[s] = ci; gr_out[s] = gr; gi_out[s] = gi;
    }
    return bad ? -19 : 0;
}

/* Working precision (double), in place on (Cr, Ci). */
int ref_zgemm_split_work(char ta, char tb, i64 m, i64 n, i64 k, const double *alpha,
                         const double *Ar, const double *Ai, i64 lda,
                         const double *Br, const double *Bi, i64 ldb, const double *beta,
                         double *Cr, double *Ci, i64 ldc)
{
    int info = check_args_z(ta, tb, m, n, k, alpha, Ar, Ai, lda, Br, Bi, ldb, beta, Cr, Ci, ldc);
    if (info) return info;
    if (m == 0 || n == 0) return 0;
    const int an = is_n(ta), bn = is_n(tb);
    const double sa = is_conj(ta) ? -1.0 : 1.0;
    const double sb = is_conj(tb) ? -1.0 : 1.0;
    const double alr = alpha[0], ali = alpha[1], ber = beta[0], bei = beta[1];
    const int use_ab = (alr != 0 || ali != 0) && k > 0;
    const int use_c = (ber != 0 || bei != 0);
    if (!use_ab && ber == 1.0 && bei == 0.0) return 0;
#pragma omp parallel for schedule(static)
    for (i64 j = 0; j < n; ++j) {
        for (i64 i = 0; i < m; ++i) {
            double pr = 0, pi = 0;
            if (use_ab) {
                for (i64 p = 0; p < k; ++p) {
                    double ar = ZA(Ar, i, p), ai = sa * ZA(Ai, i, p);
                    double br = ZB(Br, p, j), bi = sb * ZB(Bi, p, j);
                    double rr = ar * br, ii = ai * bi, ri = ar * bi, ir = ai * br;
                    pr = pr + (rr - ii);
                    pi = pi + (ri + ir);
                }
            }
            double cr = alr * pr - ali * pi;
            double ci = alr * pi + ali * pr;
            if (use_c) {
                double c0 = Cr[i + j * ldc], c1 = Ci[i + j * ldc];
                cr = cr + (ber * c0 - bei * c1);
                ci = ci + (ber * c1 + bei * c0);
            }
            Cr[i + j * ldc] = cr;
            Ci[i + j * ldc] = ci;
        }
    }
    return 0;
}


/* ------------------------------------------------------------------ */
/* LU factorisation with partial pivoting (the other LAPACK-level       */
/* driver the paper names as resting on GEMM, Abstract and Sec. 1; the  */
/* paper gives no algorithm for it, so the semantics are LAPACK's):     */
/*     P A = L U,   A m x n,  L m x min(m,n) unit lower trapezoidal,    */
/*     U min(m,n) x n upper trapezoidal,                                */
/* both overwrite A (the unit diagonal of L is not stored).  Plain      */
/* Gaussian elimination, one column at a time, in the natural order:    */
/*   for j = 0 .. min(m,n)-1                                            */
/*     p = the FIRST row index i >= j with |A(i,j)| largest             */
/*     ipiv[j] = p + 1                    (1-based, as LAPACK reports)  */
/*     if A(p,j) != 0: swap rows j and p over all n columns,            */
/*                     A(i,j) /= A(j,j) for i > j   (a true division)   */
/*     else record info = j + 1 (first such j only) and go on           */
/*     A(i,c) -= A(i,j) A(j,c)  for i > j, c > j   (multiply, then subtract) */
/* Returns info >= 0 as above, or -i for an illegal argument (m 1, n 2, */
/* A 3, lda 4, ipiv 5).                                                 */
/* ------------------------------------------------------------------ */
#define DEFINE_REF_GETRF(NAME, T, TABS)                                        \
int NAME(i64 m, i64 n, T *A, i64 lda, int *ipiv)                               \
{                                                                              \
    if (m < 0) return -1;                                                      \
    if (n < 0) return -2;                                                      \
    if (m > 0 && n > 0 && A == NULL) return -3;                                \
    if (lda < max64(1, m)) return -4;                                          \
    if (m > 0 && n > 0 && ipiv == NULL) return -5;                             \
    const i64 steps = m < n ? m : n;                                           \
    int info = 0;                                                              \
    for (i64 j = 0; j < steps; ++j) {                                          \
        i64 p = j;                                                             \
        T best = TABS(A[j + j * lda]);                                         \
        for (i64 i = j + 1; i < m; ++i) {                                      \
            const T v = TABS(A[i + j * lda]);                                  \
            if (v > best) { best = v; p = i; }                                 \
        }                                                                      \
        ipiv[j] = (int)(p + 1);                                                \
        if (A[p + j * lda] != (T)0) {                                          \
            if (p != j)                                                        \
                for (i64 c = 0; c < n; ++c) {                                  \
                    const T x = A[j + c * lda];                                \
                    A[j + c * lda] = A[p + c * lda];                           \
                    A[p + c * lda] = x;                                        \
                }                                                              \
            const T d = A[j + j * lda];                                        \
            for (i64 i = j + 1; i < m; ++i) A[i + j * lda] = A[i + j * lda] / d; \
        } else if (info == 0) {                                                \
            info = (int)(j + 1);                                               \
        }                                                                      \
        _Pragma("omp parallel for schedule(static) if ((n - j) * (m - j) > 65536)") \
        for (i64 c = j + 1; c < n; ++c) {                                      \
            const T u = A[j + c * lda];                                        \
            for (i64 i = j + 1; i < m; ++i) {                                  \
                const T prod = A[i + j * lda] * u;                             \
                A[i + c * lda] = A[i + c * lda] - prod;                        \
            }                                                                  \
        }                                                                      \
    }                                                                          \
    return info;                                                               \
}

DEFINE_REF_GETRF(ref_dgetrf, double, fabs)
DEFINE_REF_GETRF(ref_sgetrf, float, fabsf)

/* Residual of a candidate factorisation (F holding L below and U on and above
 * the diagonal, ipiv 1-based as above) against the original A0, in extended
 * precision:  R = P A0 - L U,  G = |L| |U|  (the unit diagonal of L included),
 * where P A0 is A0 with the row interchanges ipiv[0], ipiv[1], ... applied in
 * that order.  Either dense m x n (ns < 0, leading dimension m) or at ns
 * sampled entries (I[s], J[s]).  Returns 0, -i for an illegal argument (m 1,
 * n 2, A0 3, lda 4, F 5, ldf 6, ipiv 7, samples 9), or 7 if an entry of ipiv is
 * not a legal interchange (ipiv[j] outside j+1 .. m). */
#define DEFINE_REF_GETRF_RESID(NAME, T, W, WABS)                               \
int NAME(i64 m, i64 n, const T *A0, i64 lda, const T *F, i64 ldf,              \
         const int *ipiv, i64 ns, const i64 *I, const i64 *J, W *R, W *G)      \
{                                                                              \
    if (m < 0) return -1;                                                      \
    if (n < 0) return -2;                                                      \
    if (m > 0 && n > 0 && A0 == NULL) return -3;                               \
    if (lda < max64(1, m)) return -4;                                          \
    if (m > 0 && n > 0 && F == NULL) return -5;                                \
    if (ldf < max64(1, m)) return -6;                                          \
    if (m > 0 && n > 0 && ipiv == NULL) return -7;                             \
    const i64 steps = m < n ? m : n;                                           \
    for (i64 s = 0; s < (ns < 0 ? 0 : ns); ++s)                                \
        if (I[s] < 0 || I[s] >= m || J[s] < 0 || J[s] >= n) return -9;         \
    for (i64 j = 0; j < steps; ++j)                                            \
        if (ipiv[j] < j + 1 || ipiv[j] > m) return 7;                          \
    /* row i of P A0 is row src[i] of A0 */                                    \
    i64 *src = (i64 *)malloc((size_t)(m > 0 ? m : 1) * sizeof(i64));           \
    if (!src) return 1000;                                                     \
    for (i64 i = 0; i < m; ++i) src[i] = i;                                    \
    for (i64 j = 0; j < steps; ++j) {                                          \
        const i64 p = ipiv[j] - 1, x = src[j];                                 \
        src[j] = src[p];                                                       \
        src[p] = x;                                                            \
    }                                                                          \
    const i64 cnt = ns < 0 ? m * n : ns;                                       \
    _Pragma("omp parallel for schedule(dynamic, 64)")                          \
    for (i64 s = 0; s < cnt; ++s) {                                            \
        const i64 i = ns < 0 ? s % m : I[s], j = ns < 0 ? s / m : J[s];        \
        const i64 top = i < j ? i : j;          /* (L U)(i,j) = sum_{p <= min(i,j), p < steps} L(i,p) U(p,j) */ \
        W acc = (W)A0[src[i] + j * lda], mag = 0;                              \
        for (i64 p = 0; p <= top && p < steps; ++p) {                          \
            const W l = (p == i) ? (W)1 : (W)F[i + p * ldf];                   \
            const W prod = l * (W)F[p + j * ldf];                              \
            acc -= prod;                                                       \
            mag += WABS(prod);                                                 \
        }                                                                      \
        R[s] = acc;                                                            \
        G[s] = mag;                                                            \
    }                                                                          \
    free(src);                                                                 \
    return 0;                                                                  \
}

DEFINE_REF_GETRF_RESID(ref_dgetrf_resid, double, long double, fabsl)
DEFINE_REF_GETRF_RESID(ref_sgetrf_resid, float, double, fabs)
