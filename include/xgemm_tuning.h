/*
 * xgemm_tuning.h -- benchmark and tuning controls, the launch planner, the tile
 * order and the analytical kernel-selection model of the MI355X GEMM library.
 *
 * Nothing here is needed to use the BLAS-level routines of xgemm.h.  The
 * controls act on the CALLING THREAD only and are sticky: a value stays in force
 * for every later call of that thread until it is set back (-1) or
 * xgemm_tuning_reset() is called.  Code that forces anything should reset in a
 * scope guard; the library itself never changes them.
 */
#ifndef XGEMM_TUNING_H
#define XGEMM_TUNING_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Puts every control below back to its default (automatic choice) on the calling thread. */
void xgemm_tuning_reset(void);

/*
 * Benchmark/tuning control: force the tile variant used by the real GEMM
 * entry points on the calling thread.  `variant` is an index into the list
 * reported by xgemm_variant_name(); -1 restores automatic selection.
 * Returns 0, or -1 if the index is out of range.
 */
int xgemm_force_variant(int variant);

/* Benchmark/tuning control, on the calling thread, of what happens to the tiles
 * of the last, partly filled round of workgroups: -1 lets the cost model decide
 * (default); 0 runs them like the others; 1 runs them as quarter tiles in a
 * second launch wherever the shape has such a tail and a variant of half the
 * tile size exists (all real products and rank-k updates); 2..32 splits them
 * along K into that many pieces wherever the shape and workspace allow (the
 * *_ws routines).  Returns 0, or -1 for any other value.  xgemm_last_split(): pieces per tail tile used by the
 * last call on this thread (1: nothing was split). */
int xgemm_force_split(int pieces);
int xgemm_last_split(void);

/*
 * What the library would launch for a product of this shape (host only; uses
 * the CU count of the current device, 256 if there is none): out[0] tile
 * variant, out[1] pieces per split tail tile (1: none), out[2] number of tiles
 * of that variant computed whole.  If out[1] is 1 and out[2] is less than the
 * number of tiles, the remaining tiles run as four quarter tiles each, with the
 * variant of half the tile size, in a second launch (the form the last, partly
 * filled round of workgroups takes when there is no workspace to split it along K).
 * prec 'd' / 's'; uplo 0 general, 1 / 2 triangular (syrk,
 * m == n); lwork: size of the workspace the call would be given (0: none).
 * Honours xgemm_force_variant / xgemm_force_split.  Returns 0 or -i.
 */
int xgemm_plan(char prec, int uplo, int64_t m, int64_t n, int64_t k, size_t lwork, int out[3]);

/* Name of tile variant `variant` for precision `prec` ('d' or 's'), or NULL
 * past the end of the list. */
const char *xgemm_variant_name(char prec, int variant);

/* Benchmark/tuning control of xgemm_*potrf on the calling thread: panel width of
 * the look-ahead sweep.  -1: chosen from the order (default); 0: the recursion
 * alone, on the caller's stream; W > 0: panels of W columns whenever W < n.
 * Returns 0, or -1 for any other value. */
int xgemm_force_potrf_panel(int64_t width);

/* Benchmark/tuning control of xgemm_*potrf on the calling thread: the largest
 * order of a diagonal block that one workgroup factors by itself (64: one wave;
 * 128: three waves; 256: ten waves, the default, also chosen by -1); larger
 * blocks are halved.  Returns 0, or -1 for any other value. */
int xgemm_force_potrf_block(int order);

/* Benchmark/tuning control of xgemm_*getrf on the calling thread: width of the panels of the
 * right-looking sweep.  -1: chosen from the order (default); W > 0: panels of W columns.
 * Returns 0, or -1 for any other value. */
int xgemm_force_getrf_panel(int64_t width);

/* Benchmark/test control of xgemm_*getrf and xgemm_*getrf_ws on the calling thread: -1 (default) base panels
 * are held in LDS and shared by all the workgroups their rows need wherever that is possible; 0: only the
 * leaves of one workgroup each (the route that a captured call without an exchange buffer takes for panels of
 * more than 128 rows).  Returns 0, or -1 for any other value. */
int xgemm_force_getrf_shared(int mode);

/* Benchmark/test control of xgemm_*getrf_ws on the calling thread: how many polls a workgroup of a shared
 * panel waits for the others before it gives up (default 2^18, about a microsecond each).  0 makes every
 * panel shared by more than one workgroup give up at once unless all had arrived already: the way to test
 * the time-out path without holding the device.  Returns 0, or -1 for a negative value. */
int xgemm_force_getrf_spin_limit(int polls);

/* Benchmark control of xgemm_*getrf_ws on the calling thread: how long a workgroup of a shared panel waits
 * after publishing before it first looks for the others' headers resp. for the pivot row, in sleeps of 64
 * clocks (0 .. 1024 each; default 0 for both: the items are published well ahead of the first look).  Returns 0, or -1 for a value out of range. */
int xgemm_force_getrf_poll_delay(int header_sleeps, int row_sleeps);

/*
 * The workgroup -> macro-tile order the kernels use (host only, no device
 * access), for tests and for reasoning about L2 reuse: for an m x n result cut
 * into mt_m x mt_n tiles, uplo 0 (general), 1 (lower triangle) or 2 (upper
 * triangle, m == n expected for 1 and 2), returns the number of workgroups a
 * launch has and, when `out` is non-NULL, writes {tile row, tile column} of
 * workgroup b to out[2b], out[2b+1] for b < min(count, cap).  Workgroup b runs
 * on the same XCD as every workgroup b' = b (mod 8).  Exactly the tiles that intersect the requested part of C
 * appear, each once.  Returns -i for an illegal argument i.
 */
int64_t xgemm_tile_map(int uplo, int64_t m, int64_t n, int mt_m, int mt_n, int *out, int64_t cap);

/*
 * The paper's analytical kernel-selection model (host only, no device access).
 *
 * xgemm_model_outer_product_rate: Sec. 4.2.  Pipeline i retires rate[i]
 *   instructions per cycle and receives count[i] instructions per outer
 *   product; returns min_i rate[i] / count[i] over the pipelines with
 *   count[i] > 0 (infinity if there is none), in outer products per cycle.
 * xgemm_model_stalled_rate: Sec. 4.3.  A pipeline with L instructions of which
 *   n_dependent expose a latency of `latency` cycles needs W = L + n*latency;
 *   returns its instruction rate L / W (Little's law).
 * xgemm_model_n_updates: Sec. 5.4, floor((r_total - m_r*n_r/v - r_a) / r_r);
 *   r_a <= 0 means ceil(m_r / v).  Returns -1 on v <= 0 or r_r <= 0.
 * xgemm_model_predict: the model instantiated for tile variant `variant` of
 *   precision `prec` ('d' / 's') and the given transposes, per K slab:
 *   out[0] MFMAs, out[1] global loads, out[2] LDS reads, out[3] LDS writes
 *   (each per wave); out[4] matrix-pipe cycles per SIMD, out[5] LDS cycles per
 *   CU, out[6] vector-memory cycles per CU; out[7] memory instructions that must
 *   share one MFMA shadow (0: they do not fit); out[8] stall cycles of the matrix
 *   pipe per slab (Sec. 4.3's n k: one barrier per workgroup on the CU, plus the
 *   memory instructions beyond one per MFMA); out[9] predicted MFMA utilisation
 *   = out[4] / max(out[4] + out[8], out[5], out[6]); out[10] vector registers per
 *   lane (accumulators + staging + two fragment sets + 30); out[11] waves per SIMD.
 *   Returns 0; 1 if the register limit is violated; -1 bad prec, -2 bad variant,
 *   -5 out == NULL.
 * xgemm_model_efficiency: for a built variant, out[0] the fraction of the MFMA
 *   peak measured with its CUs fully occupied (the figure stored in the variant
 *   table), out[1] the model's prediction of it (transposes N, N), out[2] the one
 *   the planner prices tiles with: the model's where the two differ by at most
 *   0.025, the measured one otherwise.  Returns as xgemm_model_predict.
 * xgemm_model_enumerate: the design space the variants were taken from, in the
 *   spirit of Sec. 3.3: MFMA shape (fp64 16x16x4; fp32 32x32x2 and 16x16x4) x
 *   wave tile (MFMA tile .. 128 per side, powers of two) x waves per workgroup
 *   (1x1, 2x1, 1x2, 2x2, 4x2, 2x4) x slab depth (8, 16, 32), filtered by the
 *   register constraint of Sec. 5.4 (accumulators, one slab in flight and two
 *   fragment sets in a lane's 512 registers at the assumed occupancy), by the
 *   160 KB of LDS and by what the staging can deal to the threads, each with the
 *   utilisation the model predicts at the occupancy that fits.  Returns the
 *   number of points that pass; writes the best min(cap, count) of them to
 *   rows[12 * i + ...], best first: MFMA tile, wave tile m, n, waves along m, n,
 *   slab depth, registers, LDS bytes, workgroups per CU, predicted utilisation,
 *   macro tile m, n.  -1 bad prec, -2 cap < 0, -3 rows == NULL with cap > 0.
 */
double xgemm_model_outer_product_rate(int n_pipes, const double *rate, const double *count);
double xgemm_model_stalled_rate(double L, double n_dependent, double latency);
int xgemm_model_n_updates(int r_total, int m_r, int n_r, int v, int r_a, int r_r);
int xgemm_model_predict(char prec, int variant, char transa, char transb, double out[12]);
int xgemm_model_efficiency(char prec, int variant, double out[3]);
int xgemm_model_enumerate(char prec, int cap, double *rows);

#ifdef __cplusplus
}
#endif
#endif /* XGEMM_TUNING_H */
