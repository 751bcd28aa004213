// xgemm_zi.hip -- complex GEMM on interleaved (re, im) storage, carried by the
// real kernel: the operands are taken apart into real planes in a caller-owned
// workspace, three or four real GEMMs produce the planes of the product, and one
// pass puts  alpha * product + beta * C  back into the interleaved C.
//
//   4m:  Pr = Ar Br - Ai Bi,            Pi = Ar Bi + Ai Br          (four real products)
//   3m:  T1 = Ar Br, T2 = Ai Bi, T3 = (Ar + Ai)(Br + Bi),
//        Pr = T1 - T2,                  Pi = T3 - T1 - T2           (three real products)
//
// Fused form (method 2): ONE real product on packed operands, written straight into the interleaved C.  An
// interleaved complex matrix is a real matrix with twice the rows (re and im alternating), so
//     C~ (2m x n)  :=  A^ (2m x 2k)  B~ (2k x n)  +  beta C~,
// where B~ holds op(B) with re and im alternating along the depth and A^ holds alpha op(A) with every entry
// x = xr + i xi blown up to the 2 x 2 block [[xr, -xi], [xi, xr]]: row 2i of A^ B~ is then the real part of row i
// of the complex product and row 2i + 1 its imaginary part, 8 m n k flops like the four products of 4m, with no
// pass over C and no planes.  The two packing passes de-interleave, transpose, conjugate and scale as they go.
#include "../../include/xgemm.h"
#include "../../include/xgemm_probe.h"
#include "../../include/xgemm_tuning.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

inline bool is_n(char t) { return t == 'N' || t == 'n'; }
inline bool is_t(char t) { return t == 'T' || t == 't' || t == 'C' || t == 'c'; }
inline bool is_c(char t) { return t == 'C' || t == 'c'; }
inline int64_t max64(int64_t a, int64_t b) { return a > b ? a : b; }
constexpr int64_t DIM_MAX = 0x7fffffff;

// rows x cols complex matrix X (leading dimension ldx, in complex elements) ->
// real planes with leading dimension rows: re, im (negated when conj is set) and,
// when sum is non-NULL, re + im (of the possibly negated im).
__global__ void __launch_bounds__(256) zsplit_kernel(const double2 *X, int64_t ldx, int rows, int cols, int conj,
                                                     double *re, double *im, double *sum) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= rows) return;
    for (int j = blockIdx.y; j < cols; j += gridDim.y) {
        const double2 z = X[i + (int64_t)j * ldx];
        const double zi = conj ? -z.y : z.y;
        const int64_t o = i + (int64_t)j * rows;
        re[o] = z.x;
        im[o] = zi;
        if (sum) sum[o] = z.x + zi;
    }
}

// C (interleaved, m x n, leading dimension ldc) := alpha P + beta C with the
// planes of P given directly (three == 0: Pr = p0, Pi = p1) or through the three
// products (three != 0: Pr = p0 - p1, Pi = p2 - p0 - p1).  have_p == 0: the
// product term is absent and the planes are not read.  beta == 0: C is not read.
__global__ void __launch_bounds__(256) zmerge_kernel(double2 *C, int64_t ldc, int m, int n, const double *p0,
                                                     const double *p1, const double *p2, int three, int have_p,
                                                     double ar, double ai, double br, double bi) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= m) return;
    const bool use_c = (br != 0.0 || bi != 0.0);
    for (int j = blockIdx.y; j < n; j += gridDim.y) {
        double xr = 0.0, xi = 0.0;
        if (have_p) {
            const int64_t o = i + (int64_t)j * m;
            double pr, pi;
            if (three) {
                const double t1 = p0[o], t2 = p1[o], t3 = p2[o];
                pr = t1 - t2;
                pi = (t3 - t1) - t2;
            } else {
                pr = p0[o];
                pi = p1[o];
            }
            xr = ar * pr - ai * pi;
            xi = ar * pi + ai * pr;
        }
        double2 *c = C + i + (int64_t)j * ldc;
        if (use_c) {
            const double2 z = *c;
            xr += br * z.x - bi * z.y;
            xi += br * z.y + bi * z.x;
        }
        *c = make_double2(xr, xi);
    }
}

// Packing for the fused form, a 32 x 32 block of complex elements per workgroup through LDS so that the reads
// run along whichever index is contiguous in the source and the writes along the row index of the packed
// layout (xgemm.h: element (I, P) at [(I / 256) * 256 * kpad + P * 256 + I % 256]).
//   element (r, p) of op(X) is X[r rs + p ks] (conjugated if conj), r < rows, p < k; zero beyond.
//   EXPAND: z = alpha op(X)(r, p) goes to rows 2r, 2r + 1 and depths 2p, 2p + 1 as [[zr, -zi], [zi, zr]];
//   otherwise op(X)(r, p) goes to row r and depths 2p (re), 2p + 1 (im).
template <bool EXPAND>
__global__ void __launch_bounds__(256) zpack_kernel(const double2 *X, int64_t rs, int64_t ks, int rows, int k, int conj,
                                                    double ar, double ai, int64_t kpad, double *dst) {
    constexpr int TB = 32, PW = 256;
    __shared__ double2 tile[TB][TB + 1];     // [row][depth]
    const int tx = threadIdx.x % TB, ty = threadIdx.x / TB;
    const int r0 = blockIdx.x * TB;
    const int nby = (int)((kpad / 2 + TB - 1) / TB);
    const bool depth_runs = ks == 1 && rs != 1;
    for (int by = blockIdx.y; by < nby; by += gridDim.y) {
        const int p0 = by * TB;
        for (int j = ty; j < TB; j += 256 / TB) {
            const int rl = depth_runs ? j : tx, pl = depth_runs ? tx : j;
            const int r = r0 + rl, p = p0 + pl;
            double2 z = make_double2(0.0, 0.0);
            if (r < rows && p < k) {
                z = X[(int64_t)r * rs + (int64_t)p * ks];
                if (conj) z.y = -z.y;
                if (EXPAND) z = make_double2(ar * z.x - ai * z.y, ar * z.y + ai * z.x);
            }
            tile[rl][pl] = z;
        }
        __syncthreads();
        const int r = r0 + tx;
        for (int j = ty; j < TB; j += 256 / TB) {
            const int p = p0 + j;
            if (2 * p >= kpad) continue;
            const double2 z = tile[tx][j];
            if (EXPAND) {
                const int64_t I = 2 * (int64_t)r;
                double2 *out = reinterpret_cast<double2 *>(dst + (I / PW) * PW * kpad + (2 * (int64_t)p) * PW + I % PW);
                out[0] = z;                                   // depth 2p:      rows 2r, 2r + 1 =  zr, zi
                out[PW / 2] = make_double2(-z.y, z.x);        // depth 2p + 1:  rows 2r, 2r + 1 = -zi, zr
            } else {
                double *out = dst + ((int64_t)r / PW) * PW * kpad + (2 * (int64_t)p) * PW + r % PW;
                out[0] = z.x;
                out[PW] = z.y;
            }
        }
        __syncthreads();
    }
}

inline size_t fused_doubles(int64_t m, int64_t n, int64_t k) {
    return xgemm_pack_elems(2 * m, 2 * k) + xgemm_pack_elems(n, 2 * k);
}

size_t work_doubles(int64_t m, int64_t n, int64_t k, int method) {
    if (m <= 0 || n <= 0) return 0;
    if (method == 2) return k > 0 ? fused_doubles(m, n, k) : 0;
    const size_t planes = method == 1 ? 3 : 2;
    const size_t kk = k > 0 ? (size_t)k : 0;
    return planes * ((size_t)m * kk + kk * (size_t)n + (size_t)m * (size_t)n);
}

}  // namespace

extern "C" {

size_t xgemm_zgemm_workbytes(int64_t m, int64_t n, int64_t k, int method) {
    return work_doubles(m, n, k, method) * sizeof(double);
}

int xgemm_zgemm(char transa, char transb, int64_t m, int64_t n, int64_t k, const double alpha[2], const double *A,
                int64_t lda, const double *B, int64_t ldb, const double beta[2], double *C, int64_t ldc, int method,
                void *work, size_t lwork, void *stream) {
    if (!is_n(transa) && !is_t(transa)) return -1;
    if (!is_n(transb) && !is_t(transb)) return -2;
    if (m < 0 || m > DIM_MAX) return -3;
    if (n < 0 || n > DIM_MAX) return -4;
    if (k < 0 || k > DIM_MAX) return -5;
    if (!alpha) return -6;
    if (!beta) return -11;
    const double ar = alpha[0], ai = alpha[1], br = beta[0], bi = beta[1];
    const bool ab_read = (ar != 0.0 || ai != 0.0) && m > 0 && n > 0 && k > 0;
    const int64_t rows_a = is_n(transa) ? m : k, cols_a = is_n(transa) ? k : m;
    const int64_t rows_b = is_n(transb) ? k : n, cols_b = is_n(transb) ? n : k;
    auto misaligned = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; };
    if (ab_read && (!A || misaligned(A))) return -7;
    if (lda < max64(1, rows_a)) return -8;
    if (ab_read && (!B || misaligned(B))) return -9;
    if (ldb < max64(1, rows_b)) return -10;
    if (m > 0 && n > 0 && (!C || misaligned(C))) return -12;
    if (ldc < max64(1, m)) return -13;
    if (method < 0 || method > 2) return -14;
    if (method == 2 && (2 * m > DIM_MAX || 2 * k > DIM_MAX || 2 * ldc > DIM_MAX)) return -14;   // the real product has twice the rows and depth
    const size_t need = ab_read ? work_doubles(m, n, k, method) * sizeof(double) : 0;
    if (need > 0 && (!work || (reinterpret_cast<uintptr_t>(work) & 15u))) return -15;
    if (lwork < need) return -16;
    if (m == 0 || n == 0) return 0;
    if (!ab_read && br == 1.0 && bi == 0.0) return 0;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 blk(256);
    auto grid = [](int64_t rows, int64_t cols) {
        return dim3((unsigned)((rows + 255) / 256), (unsigned)(cols < 1024 ? cols : 1024));
    };
    double2 *Cz = reinterpret_cast<double2 *>(C);
    if (!ab_read) {
        hipLaunchKernelGGL(zmerge_kernel, grid(m, n), blk, 0, st, Cz, ldc, (int)m, (int)n, nullptr, nullptr, nullptr, 0, 0,
                           ar, ai, br, bi);
        return (int)hipGetLastError();
    }
    if (method == 2) {
        constexpr int TB = 32;
        double *const Ap = static_cast<double *>(work), *const Bp = Ap + xgemm_pack_elems(2 * m, 2 * k);
        const int64_t kpad = (2 * k + 31) / 32 * 32, nby = (kpad / 2 + TB - 1) / TB;
        const unsigned gy = (unsigned)(nby < 65535 ? nby : 65535);
        // op(A)(i, p) = A[i + p lda] (N) or A[p + i lda] (T, C);  op(B)(p, j) = B[p + j ldb] (N) or B[j + p ldb] (T, C)
        hipLaunchKernelGGL(zpack_kernel<true>, dim3((unsigned)(((2 * m + 255) / 256 * 256) / (2 * TB)), gy), blk, 0, st,
                           reinterpret_cast<const double2 *>(A), is_n(transa) ? (int64_t)1 : lda, is_n(transa) ? lda : (int64_t)1,
                           (int)m, (int)k, is_c(transa) ? 1 : 0, ar, ai, kpad, Ap);
        hipLaunchKernelGGL(zpack_kernel<false>, dim3((unsigned)(((n + 255) / 256 * 256) / TB), gy), blk, 0, st,
                           reinterpret_cast<const double2 *>(B), is_n(transb) ? ldb : (int64_t)1, is_n(transb) ? (int64_t)1 : ldb,
                           (int)n, (int)k, is_c(transb) ? 1 : 0, 1.0, 0.0, kpad, Bp);
        int rc = (int)hipGetLastError();
        if (rc) return rc;
        double beta_real = br;
        if (bi != 0.0) {
            // a complex beta cannot ride on the real product: C := beta C first, then the product is added
            hipLaunchKernelGGL(zmerge_kernel, grid(m, n), blk, 0, st, Cz, ldc, (int)m, (int)n, nullptr, nullptr, nullptr, 0, 0,
                               0.0, 0.0, br, bi);
            if ((rc = (int)hipGetLastError())) return rc;
            beta_real = 1.0;
        }
        return xgemm_dgemm_packed(2 * m, n, 2 * k, 1.0, Ap, Bp, beta_real, C, 2 * ldc, stream);
    }
    const int np = method == 1 ? 3 : 2;
    const size_t sa = (size_t)m * k, sb = (size_t)k * n, sc = (size_t)m * n;
    double *w = static_cast<double *>(work);
    double *a_re = w, *a_im = w + sa, *a_su = np == 3 ? w + 2 * sa : nullptr;
    w += np * sa;
    double *b_re = w, *b_im = w + sb, *b_su = np == 3 ? w + 2 * sb : nullptr;
    w += np * sb;
    double *p0 = w, *p1 = w + sc, *p2 = np == 3 ? w + 2 * sc : nullptr;
    hipLaunchKernelGGL(zsplit_kernel, grid(rows_a, cols_a), blk, 0, st, reinterpret_cast<const double2 *>(A), lda,
                       (int)rows_a, (int)cols_a, is_c(transa) ? 1 : 0, a_re, a_im, a_su);
    hipLaunchKernelGGL(zsplit_kernel, grid(rows_b, cols_b), blk, 0, st, reinterpret_cast<const double2 *>(B), ldb,
                       (int)rows_b, (int)cols_b, is_c(transb) ? 1 : 0, b_re, b_im, b_su);
    int rc = (int)hipGetLastError();
    if (rc) return rc;
    const char ta = is_n(transa) ? 'N' : 'T', tb = is_n(transb) ? 'N' : 'T';
    auto gemm = [&](const double *X, const double *Y, double al, double be, double *P) {
        return xgemm_dgemm(ta, tb, m, n, k, al, X, rows_a, Y, rows_b, be, P, m, stream);
    };
    if (np == 3) {
        if ((rc = gemm(a_re, b_re, 1.0, 0.0, p0))) return rc;
        if ((rc = gemm(a_im, b_im, 1.0, 0.0, p1))) return rc;
        if ((rc = gemm(a_su, b_su, 1.0, 0.0, p2))) return rc;
    } else {
        if ((rc = gemm(a_re, b_re, 1.0, 0.0, p0))) return rc;
        if ((rc = gemm(a_im, b_im, -1.0, 1.0, p0))) return rc;
        if ((rc = gemm(a_re, b_im, 1.0, 0.0, p1))) return rc;
        if ((rc = gemm(a_im, b_re, 1.0, 1.0, p1))) return rc;
    }
    hipLaunchKernelGGL(zmerge_kernel, grid(m, n), blk, 0, st, Cz, ldc, (int)m, (int)n, p0, p1, p2, np == 3 ? 1 : 0, 1, ar,
                       ai, br, bi);
    return (int)hipGetLastError();
}

}  // extern "C"
