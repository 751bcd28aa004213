/*
 * xgemm.h -- C ABI of the MI355X (gfx950) GEMM library.
 *
 * The operation is the one the paper reduces to its micro-kernel (Sec. 2.1):
 *     C += A B = sum_p a_p b_p^T     (a_p: column p of A, b_p^T: row p of B)
 * carried by the Goto/BLIS loop nest of Fig. 1, here with the column-major
 * BLAS scalars, transposes and leading dimensions around it:
 *
 *     C := alpha * op(A) * op(B) + beta * C
 *     op(A) is m x k, op(B) is k x n, C is m x n; op(X) = X or X^T.
 *
 * Conventions common to every entry point
 *   - Storage is column-major: element (i, j) of X lives at X[i + j*ldx].
 *   - Every matrix pointer is a DEVICE pointer owned by the caller.  The
 *     library never allocates, frees or keeps them.  A and B must not overlap
 *     C.  Scalars are passed by value from the host.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     only enqueue work; they do not synchronise.  All work goes to `stream`
 *     (xgemm_*potrf may also use streams of the library's between a fork from
 *     and a join to `stream`, see there; the first xgemm_*getrf of a process on
 *     a device outside a stream capture allocates an exchange buffer, which may
 *     synchronise the device that once).
 *   - trans is one of N n T t C c.  For the real routines C means T.
 *   - beta == 0: C is write-only; whatever it held (NaN, Inf) is overwritten.
 *     alpha == 0 or k == 0: A and B are not read (and may be NULL).
 *     m == 0 or n == 0, or (alpha == 0 or k == 0) and beta == 1: nothing is done.
 *     Rows m..ldc-1 of each column of C are never written.
 *   - Return value: 0 on success; -i if argument i (1-based, in the order of
 *     the prototype) is illegal, in which case nothing was enqueued; a positive
 *     value is the hipError_t of a failed launch.
 *   - Thread-safe and re-entrant.  State the library keeps, all of it per host
 *     thread unless said otherwise:
 *       . the name of the kernel variant its last call chose
 *         (xgemm_last_kernel_name) and the pieces of its last split;
 *       . the benchmark controls of xgemm_tuning.h, which stay as set until
 *         xgemm_tuning_reset() and are never touched by the routines below;
 *       . per thread and device, two streams and 23 events that xgemm_*potrf
 *         creates on its first look-ahead sweep and keeps for later calls
 *         (xgemm_release_thread_resources() destroys them);
 *       . per process and device: the exchange buffer (about 1 MiB) and the event
 *         that xgemm_*getrf allocates on its first call outside a capture and keeps,
 *         and a lock held while such a call enqueues its kernels;
 *       . per process and device, read once: the number of compute units, the
 *         address of the static scratch of xgemm_dgemm_static, and which kernels
 *         have been granted more than 64 KiB of LDS;
 *       . per process, read at load: the environment variable
 *         XGEMM_REQUIRE_ALIGNED (a test switch that sends operands that are not
 *         16-byte aligned to the element-wise fallback kernels).
 *
 * This header is the BLAS-level surface.  Benchmark and tuning controls, the
 * launch planner, the tile order and the analytical model are declared in
 * xgemm_tuning.h; the device probes in xgemm_probe.h.
 */
#ifndef XGEMM_H
#define XGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------------
 * The hot path: real GEMM in two precisions, complex GEMM on split planes as
 * four real GEMMs (with its workspace query), and two queries.
 * ------------------------------------------------------------------------ */

/*
 * Double-precision real GEMM (the micro-kernel sum of Sec. 2.1 in fp64, FP64 MFMA).
 * Illegal-argument numbering: transa 1, transb 2, m 3, n 4, k 5, alpha 6, A 7,
 * lda 8, B 9, ldb 10, beta 11, C 12, ldc 13.
 *   m, n, k >= 0;  lda >= max(1, rows of stored A) where stored A is m x k for
 *   transa = N and k x m otherwise; ldb likewise for stored B (k x n or n x k);
 *   ldc >= max(1, m).  A, B non-NULL when they are read; C non-NULL when m, n > 0.
 */
int xgemm_dgemm(char transa, char transb, int64_t m, int64_t n, int64_t k,
                double alpha, const double *A, int64_t lda,
                const double *B, int64_t ldb,
                double beta, double *C, int64_t ldc, void *stream);

/* Single-precision real GEMM; same contract as xgemm_dgemm (FP32 MFMA). */
int xgemm_sgemm(char transa, char transb, int64_t m, int64_t n, int64_t k,
                float alpha, const float *A, int64_t lda,
                const float *B, int64_t ldb,
                float beta, float *C, int64_t ldc, void *stream);

/*
 * Double-precision complex GEMM on split planes, built from the real kernel
 * (the paper's point that real GEMM carries complex GEMM, Abstract and Sec. 1;
 * the "4m" arrangement: four real products per complex product):
 *     Pr = Ar Br - Ai Bi,   Pi = Ar Bi + Ai Br,   C := alpha P + beta C.
 * Xr / Xi are the real / imaginary planes of X, each column-major with the
 * same leading dimension.  trans = C takes the conjugate transpose.
 * alpha and beta are host arrays {re, im}.
 * When alpha and beta are both real the routine is four real GEMM launches and
 * needs no workspace.  Otherwise it needs `work`: a device buffer of `lwork`
 * doubles, lwork >= xgemm_zgemm_worksize(m, n, alpha, beta); it holds Pr and Pi
 * and its contents are undefined afterwards.
 * Illegal-argument numbering: transa 1, transb 2, m 3, n 4, k 5, alpha 6, Ar 7,
 * Ai 8, lda 9, Br 10, Bi 11, ldb 12, beta 13, Cr 14, Ci 15, ldc 16, work 17,
 * lwork 18.
 */
int xgemm_zgemm_split(char transa, char transb, int64_t m, int64_t n, int64_t k,
                      const double alpha[2],
                      const double *Ar, const double *Ai, int64_t lda,
                      const double *Br, const double *Bi, int64_t ldb,
                      const double beta[2],
                      double *Cr, double *Ci, int64_t ldc,
                      double *work, int64_t lwork, void *stream);

/* Number of doubles of workspace xgemm_zgemm_split needs (0 when alpha and
 * beta are real, else 2*m*n).  Host-only; touches no device. */
size_t xgemm_zgemm_worksize(int64_t m, int64_t n, const double alpha[2], const double beta[2]);

/* Library version string (static storage). */
const char *xgemm_version(void);

/* Name of the kernel variant chosen by the last xgemm_* call on the calling
 * thread ("" before the first call, "scale" for the alpha == 0 / k == 0 path,
 * "none" for a quick return).  For benchmarks and profiles.  Static storage. */
const char *xgemm_last_kernel_name(void);

/* ------------------------------------------------------------------------
 * Beyond the hot path: the level-3 routines and drivers built on the real
 * kernel, the forms with a workspace, complex GEMM on interleaved storage.
 * ------------------------------------------------------------------------ */

/*
 * Symmetric rank-k update on the real kernel (the paper's point that the level-3
 * BLAS sit on GEMM, Abstract and Sec. 1):
 *     C := alpha * A * A^T + beta * C   (trans = N, A is n x k)
 *     C := alpha * A^T * A + beta * C   (trans = T or C, A is k x n)
 * C is n x n; only its `uplo` triangle (L: i >= j, U: i <= j, diagonal included)
 * is read and written, the other triangle is never touched.  Scalar semantics as
 * for xgemm_dgemm (beta == 0: the triangle is write-only; alpha == 0 or k == 0:
 * A is not read).  Illegal-argument numbering: uplo 1, trans 2, n 3, k 4,
 * alpha 5, A 6, lda 7, beta 8, C 9, ldc 10.  flops: n (n + 1) k.
 */
int xgemm_dsyrk(char uplo, char trans, int64_t n, int64_t k, double alpha, const double *A, int64_t lda,
                double beta, double *C, int64_t ldc, void *stream);
int xgemm_ssyrk(char uplo, char trans, int64_t n, int64_t k, float alpha, const float *A, int64_t lda,
                float beta, float *C, int64_t ldc, void *stream);

/*
 * Symmetric rank-2k update on the real kernel (two launches of the GEMM kernel in
 * triangle mode, the second accumulating onto the first):
 *     C := alpha op(A) op(B)^T + alpha op(B) op(A)^T + beta C,
 * op(X) is n x k (trans N: X; T or C: X^T, X stored k x n); only the `uplo`
 * triangle of the n x n C is read and written.  Scalar rules as for xgemm_dsyrk.
 * Illegal-argument numbering: uplo 1, trans 2, n 3, k 4, alpha 5, A 6, lda 7,
 * B 8, ldb 9, beta 10, C 11, ldc 12.  flops: 2 n (n + 1) k.
 */
int xgemm_dsyr2k(char uplo, char trans, int64_t n, int64_t k, double alpha, const double *A, int64_t lda,
                 const double *B, int64_t ldb, double beta, double *C, int64_t ldc, void *stream);
int xgemm_ssyr2k(char uplo, char trans, int64_t n, int64_t k, float alpha, const float *A, int64_t lda,
                 const float *B, int64_t ldb, float beta, float *C, int64_t ldc, void *stream);

/*
 * Symmetric matrix product on the real kernel:
 *     side L:  C := alpha A B + beta C,   A is m x m
 *     side R:  C := alpha B A + beta C,   A is n x n
 * A is symmetric and given by its `uplo` triangle; the other triangle is not
 * read.  B and C are m x n; A and B must not overlap C.  C is scaled by beta
 * first (beta == 0: written without being read), then A is halved recursively:
 * the stored off-diagonal block enters two GEMMs (as it is and transposed),
 * diagonal blocks of order <= 64 are mirrored into full blocks by a small
 * kernel.  Every element satisfies the product bound with k = m (L) or n (R).
 * Illegal-argument numbering: side 1, uplo 2, m 3, n 4, alpha 5, A 6, lda 7,
 * B 8, ldb 9, beta 10, C 11, ldc 12.  flops: 2 m^2 n (L) or 2 m n^2 (R).
 */
int xgemm_dsymm(char side, char uplo, int64_t m, int64_t n, double alpha, const double *A, int64_t lda,
                const double *B, int64_t ldb, double beta, double *C, int64_t ldc, void *stream);
int xgemm_ssymm(char side, char uplo, int64_t m, int64_t n, float alpha, const float *A, int64_t lda,
                const float *B, int64_t ldb, float beta, float *C, int64_t ldc, void *stream);

/*
 * Triangular solve with many right-hand sides on the real kernel (level-3 BLAS
 * above GEMM, Abstract and Sec. 1):
 *     side L:  op(T) X = alpha B,   T is m x m
 *     side R:  X op(T) = alpha B,   T is n x n
 * B (m x n) is overwritten by X.  T is triangular: only its `uplo` triangle is
 * read (the other one may hold anything); diag U takes a unit diagonal and does
 * not read the stored one.  alpha == 0 gives X = 0 without reading T or B.
 * T is halved recursively; the halves are coupled by GEMMs with the
 * off-diagonal block (alpha -1, beta 1), diagonal blocks of order <= 64 are
 * solved by substitution, so every element of X comes out of a sum of at most
 * dim products plus one division (multiplication by the reciprocal of the
 * diagonal entry) and satisfies the componentwise residual bound
 *     |alpha B - op(T) X| <= 4 dim u (|alpha B| + |op(T)| |X|),  dim = m or n.
 * T must not overlap B.  No singularity check.  Illegal-argument numbering:
 * side 1, uplo 2, transa 3, diag 4, m 5, n 6, alpha 7, A 8, lda 9, B 10, ldb 11.
 * flops: m^2 n (side L) or m n^2 (side R).
 */
int xgemm_dtrsm(char side, char uplo, char transa, char diag, int64_t m, int64_t n, double alpha,
                const double *A, int64_t lda, double *B, int64_t ldb, void *stream);
int xgemm_strsm(char side, char uplo, char transa, char diag, int64_t m, int64_t n, float alpha,
                const float *A, int64_t lda, float *B, int64_t ldb, void *stream);

/*
 * Triangular matrix product on the real kernel, in place:
 *     side L:  B := alpha op(T) B,   T is m x m
 *     side R:  B := alpha B op(T),   T is n x n
 * Conventions, argument numbering and flop count as for xgemm_dtrsm (only the
 * `uplo` triangle of T is read, diag U implies ones, alpha == 0 gives B = 0
 * without reading T or B, T must not overlap B).  Same recursive organisation:
 * the halves of T are coupled by GEMMs with the off-diagonal block, diagonal
 * blocks of order <= 64 are multiplied by a small kernel.  Every element is a
 * sum of at most dim products in some order, so it satisfies the product bound
 *     |B_out - alpha op(T) B| <= 4 dim u |alpha| |op(T)| |B|.
 */
int xgemm_dtrmm(char side, char uplo, char transa, char diag, int64_t m, int64_t n, double alpha,
                const double *A, int64_t lda, double *B, int64_t ldb, void *stream);
int xgemm_strmm(char side, char uplo, char transa, char diag, int64_t m, int64_t n, float alpha,
                const float *A, int64_t lda, float *B, int64_t ldb, void *stream);

/*
 * Cholesky factorisation on the level-3 routines (a LAPACK-level driver of the
 * kind the paper names as the reason for a fast GEMM, Sec. 1):
 *     uplo L:  A = L L^T, the lower triangle of A is overwritten by L
 *     uplo U:  A = U^T U, the upper triangle of A is overwritten by U
 * A is n x n symmetric positive definite, given by its `uplo` triangle; the
 * other triangle is neither read nor written.  Recursive: factor the leading
 * half, solve for the off-diagonal block (xgemm_*trsm), update the trailing
 * half (xgemm_*syrk), factor it; diagonal blocks of order <= 256 are factored by
 * one workgroup.  Blocks of order 3072 to 16384 (fp32: from 3072 on; larger
 * fp64 matrices are halved down to that first) are instead swept right-looking
 * over panels of 256 or 512 columns with look-ahead: the factorisation of the
 * next panel (the recursion above) and the solves and updates that only the
 * next panel needs run on two streams of the library's beside the trailing
 * update of the current one.  Those streams (per host thread and device,
 * created by the first such call and kept) branch off `stream` at the start of
 * the call and are joined to it before the call returns, so the call orders
 * like work on `stream` alone.  While `stream` is being captured into a graph
 * the same kernels are all enqueued on `stream` itself, in an order that gives
 * the same bits.
 * `info` is a DEVICE int written on the stream: 0 on success,
 * j > 0 if the leading minor of order j is not positive definite (the factor is
 * then undefined from column j on, and only the first failure is recorded).
 * The computed factor satisfies |A - L L^T| <= 4 n u |L| |L|^T on the triangle.
 * Returns 0, -i for an illegal argument (uplo 1, n 2, A 3, lda 4, info 5) or a
 * hipError_t.  flops: n^3 / 3.
 */
int xgemm_dpotrf(char uplo, int64_t n, double *A, int64_t lda, int *info, void *stream);
int xgemm_spotrf(char uplo, int64_t n, float *A, int64_t lda, int *info, void *stream);

/*
 * LU factorisation with partial pivoting on the level-3 routines (the other LAPACK-level
 * driver of the kind the paper names as the reason for a fast GEMM, Abstract and Sec. 1;
 * the paper gives no algorithm for it, the semantics are LAPACK's getrf):
 *     P A = L U,   A is m x n,
 * L (m x min(m,n), unit lower trapezoidal, its diagonal not stored) and U (min(m,n) x n,
 * upper trapezoidal) overwrite A.  ipiv (DEVICE, min(m,n) ints) receives the interchanges,
 * 1-based: at step j, row j changed places with row ipiv[j] >= j; the pivot of a column is
 * the first of its entries of largest magnitude.  `info` (DEVICE int, written on the
 * stream): 0, or j > 0 if U(j,j) is exactly zero (the first such j; the factorisation is
 * completed all the same, as in LAPACK).  Every multiplier satisfies |L(i,j)| <= 1 and the
 * factors satisfy |P A - L U| <= 4 min(m,n) u |L| |U| element by element.
 *
 * How it runs.  The matrix is halved recursively by columns onto xgemm_*trsm and xgemm_*gemm
 * down to base panels of 128 columns; a base panel's interchanges are applied to the other
 * columns by a kernel of their own.  A base panel is factored by all the workgroups its rows
 * need at once: its rows are dealt to workgroups in stripes of 128, each stripe stays in the
 * LDS of its workgroup for the whole panel, and the pivot of a column is agreed by every
 * workgroup alike from the candidates (value, row and the whole candidate row) that all of
 * them publish in an exchange buffer.  That buffer (about 1 MiB) is one per device, allocated
 * by the first call that needs it and kept for the life of the process.
 * The workgroups of such a panel wait for each other (the only place in the library where a
 * workgroup waits for another), so all of them must be resident together: the library never
 * asks for more than one per compute unit, and it orders every factorisation of this kind on
 * a device behind the one before it, whichever host thread and stream it comes from (an
 * event; calls on different streams therefore do not overlap each other).  Every wait is
 * bounded: a workgroup that does not see the others within a few tenths of a second gives
 * up, the others follow, and *info becomes -1 (A is then partly factored and must be
 * discarded); that can only happen when other work holds the device's compute units for
 * that long.
 * Where that cannot be done (the stream is being captured, where nothing may be allocated and
 * no event of the library's waited for; a panel of more than 128 rows per compute unit of the
 * device; the allocation failed) a base panel is halved further down to leaves of 8 columns
 * that one workgroup each factors on its own, as every panel of at most 128 rows is anyway.
 * Returns 0, -i for an illegal argument (m 1, n 2, A 3, lda 4, ipiv 5, info 6)
 * or a hipError_t.  flops: m n^2 - n^3 / 3 for m >= n (2 n^3 / 3 when square).
 */
int xgemm_dgetrf(int64_t m, int64_t n, double *A, int64_t lda, int *ipiv, int *info, void *stream);
int xgemm_sgetrf(int64_t m, int64_t n, float *A, int64_t lda, int *ipiv, int *info, void *stream);

/*
 * The same factorisation with a caller-owned exchange buffer: for callers that keep device memory
 * under their own control, and the only way to get shared panels into a captured graph.
 *   work : device buffer, 16-byte aligned, lwork >= xgemm_getrf_workspace_bytes() (about 1 MiB); its
 *          contents need no preparation and are undefined afterwards.  Calls that share it must not
 *          overlap in time.  NULL or too small: the call runs exactly as xgemm_*getrf.
 * Outside a capture these calls take part in the order described above.  A captured call cannot (it may
 * not wait for an event recorded outside its capture): two factorisations with shared panels that run at
 * the same time on one device can each hold the compute units the other waits for and both time out, so
 * a graph that holds one must not be replayed beside another such factorisation.
 * Same semantics, same pivot rule, same bits as xgemm_*getrf where that uses shared panels too.
 * Returns as xgemm_*getrf, and -7 for a work that is not 16-byte aligned.
 */
size_t xgemm_getrf_workspace_bytes(void);
int xgemm_dgetrf_ws(int64_t m, int64_t n, double *A, int64_t lda, int *ipiv, int *info, void *work, size_t lwork,
                    void *stream);
int xgemm_sgetrf_ws(int64_t m, int64_t n, float *A, int64_t lda, int *ipiv, int *info, void *work, size_t lwork,
                    void *stream);

/*
 * GEMM and SYRK with a caller-owned workspace, which lets the library
 * cut the tiles of the last, partly filled round of workgroups along K (the k_c
 * loop of Fig. 1 moved across workgroups for those tiles only): each piece
 * leaves its partial sums in the workspace, the piece that finishes last adds
 * them in a fixed order and writes C, so results do not depend on timing and
 * satisfy the same error bound.  Whether and how far to split is decided by the
 * cost model from the shape; shapes that fill their rounds run exactly as in
 * the plain routines.
 *   work : device buffer, 16-byte aligned, lwork bytes; xgemm_workspace_bytes()
 *          is the size that never limits the split (8 KiB of counters + 64 MiB).
 *          Smaller buffers split less; NULL or lwork <= 8 KiB: never split.
 *          Before its first use the first 8 KiB must be zero
 *          (xgemm_workspace_init); every call leaves them zero again.  Calls
 *          that share a workspace must be ordered on one stream (or otherwise
 *          not overlap); its other contents are undefined after a call.
 * Illegal-argument numbering as in the plain routines, then work (14 for gemm,
 * 11 for syrk; reported when it is not 16-byte aligned).
 */
size_t xgemm_workspace_bytes(void);
/* Clears the counters at the start of `work` on `stream` (a kernel launch).
 * Returns 0, -1 (work NULL or misaligned), -2 (lwork < 8 KiB) or a hipError_t. */
int xgemm_workspace_init(void *work, size_t lwork, void *stream);
int xgemm_dgemm_ws(char transa, char transb, int64_t m, int64_t n, int64_t k,
                   double alpha, const double *A, int64_t lda, const double *B, int64_t ldb,
                   double beta, double *C, int64_t ldc, void *work, size_t lwork, void *stream);
int xgemm_sgemm_ws(char transa, char transb, int64_t m, int64_t n, int64_t k,
                   float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                   float beta, float *C, int64_t ldc, void *work, size_t lwork, void *stream);
int xgemm_dsyrk_ws(char uplo, char trans, int64_t n, int64_t k, double alpha, const double *A, int64_t lda,
                   double beta, double *C, int64_t ldc, void *work, size_t lwork, void *stream);
int xgemm_ssyrk_ws(char uplo, char trans, int64_t n, int64_t k, float alpha, const float *A, int64_t lda,
                   float beta, float *C, int64_t ldc, void *work, size_t lwork, void *stream);

/*
 * xgemm_dgemm_ws for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * split tail, with the workspace taken from a fixed array of
 * XGEMM_STATIC_SCRATCH_BYTES that is part of the library's code object (every
 * device the library runs on holds its own copy from load until the process
 * ends).  The call allocates and frees nothing, in the library or through the
 * runtime; the caller passes only the operands.  Arguments, numbering, results
 * and error bound are those of xgemm_dgemm_ws given a full-size workspace: the
 * same plan, hence the same bits.
 *   - A shape whose split tail would use more than the array holds (counters +
 *     pieces * tail tiles * 128 KiB) is refused with XGEMM_E_SCRATCH and nothing
 *     is enqueued; xgemm_dgemm, which needs no workspace, serves it.
 *   - The counters in the array are cleared by a kernel on `stream` at the start
 *     of every call that splits (no memset, so the call can be captured).
 *   - All calls on one device share that device's array: calls that may overlap
 *     in time (different streams without ordering, several host threads) race on
 *     it and give undefined results.  Order them, or use xgemm_dgemm_ws with a
 *     workspace per stream.
 *   - The first call on a device looks the array's address up in the runtime;
 *     make that call outside a stream capture.
 * Returns 0, -i, XGEMM_E_SCRATCH or a hipError_t.
 */
#define XGEMM_STATIC_SCRATCH_BYTES (8192 + (32 << 20))
#define XGEMM_E_SCRATCH (-1000)
int xgemm_dgemm_static(char transa, char transb, int64_t m, int64_t n, int64_t k,
                       double alpha, const double *A, int64_t lda, const double *B, int64_t ldb,
                       double beta, double *C, int64_t ldc, void *stream);

/*
 * Packed operands (the explicit packing of Fig. 1 and Sec. 2.2, done once in device memory for operands
 * that enter several products).  xgemm_*pack_a writes op(A) (m x k), xgemm_*pack_b writes op(B) (k x n) into a
 * buffer of xgemm_pack_elems(m, k) resp. xgemm_pack_elems(n, k) elements, 16-byte aligned, in panels of 256 rows
 * of op(A) (columns of op(B)), depth-major inside a panel:
 *     element (i, p)  at  [(i / 256) * 256 * Kpad + p * 256 + i % 256],   Kpad = k rounded up to 32,
 * zero beyond the matrix.  The transpose (N, T; C is T) and the leading dimension of the source are absorbed:
 * xgemm_*gemm_packed computes  C := alpha op(A) op(B) + beta C  from the two buffers alone, with every slab of
 * every tile a run of whole 16-byte vectors.  A packed operand may be used by any number of products; it must
 * not overlap C.  Same element-wise result as xgemm_*gemm on the unpacked operands wherever both take the same
 * tile variant (the sums run over k in the same order).
 * Illegal-argument numbering: pack_a: transa 1, m 2, k 3, A 4, lda 5, Ap 6;  pack_b: transb 1, k 2, n 3, B 4,
 * ldb 5, Bp 6;  gemm_packed: m 1, n 2, k 3, Ap 5, Bp 6, C 8, ldc 9.  Positive: a HIP error.
 */
size_t xgemm_pack_elems(int64_t rows, int64_t k);
int xgemm_dpack_a(char transa, int64_t m, int64_t k, const double *A, int64_t lda, double *Ap, void *stream);
int xgemm_dpack_b(char transb, int64_t k, int64_t n, const double *B, int64_t ldb, double *Bp, void *stream);
int xgemm_spack_a(char transa, int64_t m, int64_t k, const float *A, int64_t lda, float *Ap, void *stream);
int xgemm_spack_b(char transb, int64_t k, int64_t n, const float *B, int64_t ldb, float *Bp, void *stream);
int xgemm_dgemm_packed(int64_t m, int64_t n, int64_t k, double alpha, const double *Ap, const double *Bp, double beta,
                       double *C, int64_t ldc, void *stream);
int xgemm_sgemm_packed(int64_t m, int64_t n, int64_t k, float alpha, const float *Ap, const float *Bp, float beta,
                       float *C, int64_t ldc, void *stream);

/*
 * Double-precision complex GEMM on interleaved storage (the BLAS layout: element
 * (i, j) of X is the pair X[2*(i + j*ldx)], X[2*(i + j*ldx) + 1]; leading
 * dimensions count complex elements; A, B, C 16-byte aligned), built from the
 * real kernel:
 *     C := alpha op(A) op(B) + beta C,   op(X) = X, X^T or X^H (trans N, T, C).
 * The operands are taken apart into real planes in `work`, real GEMMs produce
 * the planes of the product, and one pass merges alpha * product + beta * C
 * into C.
 *   method 0 ("4m"): four real products, Pr = Ar Br - Ai Bi, Pi = Ar Bi + Ai Br;
 *            each plane within 8 k u of its own sum of magnitudes.
 *   method 1 ("3m"): three real products, T1 = Ar Br, T2 = Ai Bi,
 *            T3 = (Ar + Ai)(Br + Bi), Pr = T1 - T2, Pi = T3 - T1 - T2: a quarter
 *            fewer flops, but the imaginary part is only accurate relative to
 *            (|Ar| + |Ai|)(|Br| + |Bi|), i.e. to the magnitudes of both planes.
 *   method 2 (fused): one real product written straight into C.  C as a real matrix has
 *            twice the rows (re, im alternating); alpha op(A) is packed with every entry
 *            x blown up to [[xr, -xi], [xi, xr]] (2m x 2k), op(B) with re, im alternating
 *            along the depth (2k x n), both in the layout of xgemm_dpack_a / _b, and
 *            xgemm_dgemm_packed(2m, n, 2k) adds their product to beta C (a complex beta
 *            scales C in a pass of its own first).  8 m n k flops, the same sums of
 *            magnitudes per plane as 4m, no planes and no pass over C after the product.
 *            Needs 2 m, 2 k and 2 ldc within 2^31 - 1 (else -14).
 * work: device buffer, 16-byte aligned, lwork >= xgemm_zgemm_workbytes(m, n, k,
 * method) bytes (methods 0, 1: 2 or 3 planes each of A, B and the product; method 2:
 * the two packed operands, xgemm_pack_elems(2m, 2k) + xgemm_pack_elems(n, 2k) doubles); contents undefined
 * afterwards; not needed when alpha == 0 or k == 0.  alpha, beta: host {re, im}.
 * Illegal-argument numbering: transa 1, transb 2, m 3, n 4, k 5, alpha 6, A 7,
 * lda 8, B 9, ldb 10, beta 11, C 12, ldc 13, method 14, work 15, lwork 16.
 * flops counted as 8 m n k for both methods.
 */
int xgemm_zgemm(char transa, char transb, int64_t m, int64_t n, int64_t k, const double alpha[2],
                const double *A, int64_t lda, const double *B, int64_t ldb, const double beta[2],
                double *C, int64_t ldc, int method, void *work, size_t lwork, void *stream);
size_t xgemm_zgemm_workbytes(int64_t m, int64_t n, int64_t k, int method);

/*
 * Destroys the streams and events that xgemm_*potrf keeps for the calling thread on
 * the current device (after waiting for the work on them); the next call that needs
 * them creates them again.  For threads that end, and for callers that count handles.
 * Must not be called while a call of this thread is being captured.  Returns 0 or a
 * hipError_t.
 */
int xgemm_release_thread_resources(void);

#ifdef __cplusplus
}
#endif
#endif /* XGEMM_H */
