/*
 * xgemm_probe.h -- device probes of the MI355X GEMM library: small kernels that
 * measure the machine (matrix-core peak, instruction latencies) or report how it
 * places work (accumulator layout, workgroup placement).  Used by the benchmark
 * and by the tests that check the assumptions the kernels are built on; not
 * needed to use the routines of xgemm.h.  Pointers are DEVICE pointers owned by
 * the caller; `stream` as in xgemm.h.
 */
#ifndef XGEMM_PROBE_H
#define XGEMM_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * MFMA-only micro-benchmark (confirms the matrix-core peak that percentages
 * are quoted against): launches `blocks` workgroups of 256 threads, each wave
 * issuing `iters` rounds of back-to-back register-resident MFMAs with no
 * memory traffic in the loop: 16 FP64 16x16x4 per round for prec 'd', 8 FP32
 * 32x32x2 per round for 's'.  `sink` is a device buffer of at least blocks*256
 * elements of that precision, written once at the end.  Returns 0 or a
 * hipError_t.  flops per launch = blocks * 4 waves * iters * 32768 for both
 * precisions (16 * 2*16*16*4 = 8 * 2*32*32*2 = 32768).
 */
int xgemm_mfma_peak_probe(char prec, int blocks, int iters, void *sink, void *stream);

/*
 * Writes the register layout of one MFMA result to `out` (device, 64*R ints
 * where R = 4 for 'd', 16 for 's'): out[lane*R + r] = 256*i + j for the matrix
 * element D(i, j) held by lane `lane`, register r, found by multiplying one-hot
 * operands.  Used by the tests to confirm the accumulator layout the kernels
 * assume.  Returns 0 or a hipError_t.
 */
int xgemm_mfma_layout_probe(char prec, int *out, void *stream);

/*
 * Latency probe: what a dependent chain of instructions costs a lone wave, the
 * device's counterpart of the latency column of the paper's micro-architecture
 * table (Sec. 4.3, the k of W = L + n k).  One wave runs `iters` rounds of eight
 * chains and writes the elapsed ticks of the 100 MHz real-time counter (10 ns each)
 * to out[0..7] (device, 8 x int64); per round the chains hold
 *   0: 8 FP64 fused multiply-adds       1: 8 FP32 fused multiply-adds
 *   2: 8 FP64 reciprocal square roots, each fed through one add
 *   3: 4 LDS round trips (write, then read what another lane wrote)
 *   4: 4 FP64 16x16x4 matrix instructions accumulating into one tile
 *   5: 4 x (matrix instruction, vector instruction on its result, next matrix instruction)
 *   6: 8 x (lane read into scalar registers, vector instruction that uses them)
 *   7: 4 FP32 32x32x2 matrix instructions accumulating into one tile
 * so that ns per instruction = 10 * out[i] / (iters * count_i).  `sink` (device,
 * 64 doubles) receives the chains' values so that nothing is optimised away.
 * Returns 0 or a hipError_t (iters must be in 1 .. 2^20).
 */
int xgemm_latency_probe(long long *out, double *sink, int iters, void *stream);

/*
 * Placement probe: launches `blocks` workgroups of 256 threads, each asking for
 * `lds_bytes` of LDS (0..163840) and staying resident for a fixed ~200k cycles,
 * and writes 4 unsigned ints per wave to `out` (device, 16*blocks values):
 * {HW_ID register, XCC_ID register, workgroup index, wave index in workgroup}.
 * Shows which XCD, CU, SIMD and wave slot the hardware dispatcher gives to
 * consecutive workgroups (the assumption behind the XCD-aware tile order).
 * Returns 0 or a hipError_t.
 */
int xgemm_hwid_probe(int blocks, int lds_bytes, unsigned *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* XGEMM_PROBE_H */
