// xgemm_d.hip -- fp64 kernel instantiations (FP64 MFMA 16x16x4).
#include "tables.h"

namespace xg {

// name: MT_M x MT_N x KT, waves along m x n, waves per SIMD the register budget allows
using D_128x128x16 = TileCfg<double, 128, 128, 16, 2, 2, 2>;
using D_128x128x8 = TileCfg<double, 128, 128, 8, 2, 2, 2>;
using D_256x128x8 = TileCfg<double, 256, 128, 8, 4, 2, 2>;
using D_64x64x16 = TileCfg<double, 64, 64, 16, 2, 2, 2>;

#define XG_ENTRY(T, CFG, NAME) {NAME, CFG::MT_M, CFG::MT_N, &launch_cfg<T, CFG>}

const VariantEntry<double> *d_variant_table(int *n) {
    static const VariantEntry<double> table[] = {
    XG_ENTRY(double, D_128x128x16, "d_128x128x16_w2x2"),
    XG_ENTRY(double, D_128x128x8, "d_128x128x8_w2x2"),
    XG_ENTRY(double, D_256x128x8, "d_256x128x8_w4x2"),
    XG_ENTRY(double, D_64x64x16, "d_64x64x16_w2x2"),
    };
    *n = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}

}  // namespace xg
