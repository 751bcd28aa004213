// xgemm_pack.hip -- explicit packing of an operand into panel-major memory: the step the paper's Fig. 1 draws
// as blocked arrows (Sec. 2.2: blocks of A and B are copied into contiguous buffers laid out in the order the
// micro-kernel reads them), done once in HBM for operands that are used by several products.
//
// Layout (the same for op(A), indexed (row i, depth p), and for op(B), indexed (column j, depth p)): panels of
// PACK_W = 256 rows; inside a panel, depth-major with the 256 rows of one depth step contiguous:
//     element (i, p)  at  [(i / 256) * 256 * Kpad + p * 256 + i % 256],   Kpad = k rounded up to 32,
// zero where i or p lies beyond the matrix.  A slab of any tile variant (256, 128, 64 or 32 rows by 8, 16 or 32
// depth steps) is then whole runs of 16-byte vectors whatever the transpose and leading dimension of the source
// were, and the product kernel reads it as an MN-contiguous operand with leading dimension 256.
#include "../../include/xgemm.h"
#include "tables.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int PW = xg::PACK_W, KR = 32, TILE = 64;
static_assert(PW % TILE == 0, "a 64 x 64 block of the copy lies inside one panel");
constexpr int64_t DIM_MAX = 0x7fffffff;

inline int64_t round_up(int64_t x, int64_t to) { return (x + to - 1) / to * to; }

// 64 rows x 64 depth steps per workgroup through LDS, so that both the reads (along whichever index is
// contiguous in the source: rs == 1 rows, ks == 1 depth) and the writes (along rows) are whole lines.
template <typename T>
__global__ void __launch_bounds__(256) pack_kernel(const T *src, int64_t rs, int64_t ks, int rows, int k, int64_t kpad, T *dst) {
    __shared__ T tile[TILE][TILE + 1];     // [row][depth]
    const int tx = threadIdx.x % TILE, ty = threadIdx.x / TILE;
    const int r0 = blockIdx.x * TILE;
    const int nby = (int)((kpad + TILE - 1) / TILE);
    const bool depth_runs = ks == 1 && rs != 1;
    for (int by = blockIdx.y; by < nby; by += gridDim.y) {
        const int p0 = by * TILE;
        for (int j = ty; j < TILE; j += 256 / TILE) {
            const int il = depth_runs ? j : tx, pl = depth_runs ? tx : j;
            const int i = r0 + il, p = p0 + pl;
            tile[il][pl] = (i < rows && p < k) ? src[(int64_t)i * rs + (int64_t)p * ks] : T(0);
        }
        __syncthreads();
        const int i = r0 + tx;
        T *const out = dst + (int64_t)(i / PW) * PW * kpad + i % PW;
        for (int j = ty; j < TILE; j += 256 / TILE) {
            const int p = p0 + j;
            if (p < kpad) out[(int64_t)p * PW] = tile[tx][j];
        }
        __syncthreads();
    }
}

// op(X) has `rows` rows (its m or n index) and depth k; element (i, p) of it is src[i * rs + p * ks]
template <typename T> int pack_impl(int64_t rows, int64_t k, const T *src, int64_t rs, int64_t ks, T *dst, void *stream) {
    if (rows == 0 || k == 0) return 0;
    const int64_t kpad = round_up(k, KR), rpad = round_up(rows, PW);
    const int64_t nby = (kpad + TILE - 1) / TILE;
    const dim3 grid((unsigned)(rpad / TILE), (unsigned)(nby < 65535 ? nby : 65535));
    hipLaunchKernelGGL(pack_kernel<T>, grid, dim3(256), 0, static_cast<hipStream_t>(stream), src, rs, ks, (int)rows, (int)k, kpad, dst);
    return (int)hipGetLastError();
}

inline bool is_n(char t) { return t == 'N' || t == 'n'; }
inline bool is_t(char t) { return t == 'T' || t == 't' || t == 'C' || t == 'c'; }

// stored: the matrix as stored has `srows` rows; op(X)(i, p) = X[i + p ld] when `rows_run` (the op's row index
// runs down the stored columns), X[p + i ld] otherwise
template <typename T>
int pack_checked(char trans, bool a_side, int64_t d1, int64_t d2, const T *X, int64_t ld, T *Xp, void *stream) {
    if (!is_n(trans) && !is_t(trans)) return -1;
    if (d1 < 0 || d1 > DIM_MAX) return -2;
    if (d2 < 0 || d2 > DIM_MAX) return -3;
    // A: op(A) is m x k = d1 x d2, stored m x k (N) or k x m (T);  B: op(B) is k x n = d1 x d2, stored k x n (N) or n x k (T)
    const int64_t stored_rows = is_n(trans) ? d1 : d2;
    const int64_t rows = a_side ? d1 : d2, k = a_side ? d2 : d1;
    if (rows > 0 && k > 0 && !X) return -4;
    if (ld < (stored_rows > 1 ? stored_rows : 1)) return -5;
    if (rows > 0 && k > 0 && !Xp) return -6;
    // the op's row index (m for A, n for B) runs down the stored columns for A with N and for B with T
    const bool rows_run = a_side ? is_n(trans) : is_t(trans);
    return pack_impl<T>(rows, k, X, rows_run ? 1 : ld, rows_run ? ld : 1, Xp, stream);
}

}  // namespace

extern "C" {

size_t xgemm_pack_elems(int64_t rows, int64_t k) {
    if (rows <= 0 || k <= 0 || rows > DIM_MAX || k > DIM_MAX) return 0;
    return (size_t)round_up(rows, PW) * (size_t)round_up(k, KR);
}

int xgemm_dpack_a(char transa, int64_t m, int64_t k, const double *A, int64_t lda, double *Ap, void *stream) {
    return pack_checked<double>(transa, true, m, k, A, lda, Ap, stream);
}
int xgemm_dpack_b(char transb, int64_t k, int64_t n, const double *B, int64_t ldb, double *Bp, void *stream) {
    return pack_checked<double>(transb, false, k, n, B, ldb, Bp, stream);
}
int xgemm_spack_a(char transa, int64_t m, int64_t k, const float *A, int64_t lda, float *Ap, void *stream) {
    return pack_checked<float>(transa, true, m, k, A, lda, Ap, stream);
}
int xgemm_spack_b(char transb, int64_t k, int64_t n, const float *B, int64_t ldb, float *Bp, void *stream) {
    return pack_checked<float>(transb, false, k, n, B, ldb, Bp, stream);
}

}  // extern "C"
