// tables.h -- variant tables defined by the per-precision translation units.
#pragma once
#include "variants.hip.h"

namespace xg {
// Each returns its table and writes the number of entries to *n.
const VariantEntry<double> *d_variant_table(int *n);
const VariantEntry<float> *s_variant_table(int *n);
}  // namespace xg
