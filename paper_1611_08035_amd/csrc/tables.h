// tables.h -- variant tables defined by the per-precision translation units.
#pragma once
#include "variants.hip.h"

namespace xg {
// Each returns its table and writes the number of entries to *n.
const VariantEntry<double> *d_variant_table(int *n);
const VariantEntry<float> *s_variant_table(int *n);

// C += alpha op(A) op(B) with a depth range per tile (GemmArgs::kcut, kaxis, kblk, reverse): not
// part of the C interface, used by the symmetric product.  Returns as the real products do.
int gemm_cut(char ta, char tb, int64_t m, int64_t n, int64_t k, double alpha, const double *A, int64_t lda,
             const double *B, int64_t ldb, double *C, int64_t ldc, void *stream, int kcut, int kaxis, int kblk);
int gemm_cut(char ta, char tb, int64_t m, int64_t n, int64_t k, float alpha, const float *A, int64_t lda,
             const float *B, int64_t ldb, float *C, int64_t ldc, void *stream, int kcut, int kaxis, int kblk);

// Full-occupancy efficiency of a variant as the planner takes it: the analytical model's prediction where that
// is within its tolerance of the measured figure in the table, the measured figure otherwise.
double planner_eff(const VariantEntry<double> &v);
double planner_eff(const VariantEntry<float> &v);

// Puts the benchmark controls of the factorisation (panel width, block order) back to automatic on the
// calling thread; defined beside them.
void reset_l3_tuning();
void reset_lu_tuning();
}  // namespace xg
