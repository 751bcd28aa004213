// xgemm_d.hip -- fp64 kernel instantiations (FP64 MFMA 16x16x4).
#include "tables.h"

namespace xg {

// name: MT_M x MT_N x KT, waves along m x n, waves per SIMD the register budget allows
using D_128x128x16 = TileCfg<double, 128, 128, 16, 2, 2, 2>;
using D_128x128x8 = TileCfg<double, 128, 128, 8, 2, 2, 2>;
using D_256x128x8 = TileCfg<double, 256, 128, 8, 4, 2, 2>;
using D_64x64x16 = TileCfg<double, 64, 64, 16, 2, 2, 2, 2>;   // slabs asked for two ahead: a slab of this tile is shorter than a memory round trip
using D_128x64x16 = TileCfg<double, 128, 64, 16, 2, 2, 2>;
using D_64x128x16 = TileCfg<double, 64, 128, 16, 2, 2, 2>;
using D_32x32x16 = TileCfg<double, 32, 32, 16, 2, 2, 2, 2>;   // one matrix-instruction tile per wave: for products too small to fill the device with larger tiles

#define XG_ENTRY(T, CFG, NAME, WGS, EFF, LONE) {NAME, CFG::MT_M, CFG::MT_N, CFG::KT, CFG::WGM, CFG::WGN, WGS, EFF, LONE, false, &launch_cfg<T, CFG, false>}
// the same with the split-tail kernels built as well
#define XG_ENTRY_SPLIT(T, CFG, NAME, WGS, EFF, LONE) {NAME, CFG::MT_M, CFG::MT_N, CFG::KT, CFG::WGM, CFG::WGN, WGS, EFF, LONE, true, &launch_cfg<T, CFG, true>}

const VariantEntry<double> *d_variant_table(int *n) {
    static const VariantEntry<double> table[] = {
    XG_ENTRY_SPLIT(double, D_128x128x16, "d_128x128x16_w2x2", 2, 0.975f, 0.94f),
    XG_ENTRY(double, D_128x128x8, "d_128x128x8_w2x2", 2, 0.93f, 0.90f),
    XG_ENTRY(double, D_256x128x8, "d_256x128x8_w4x2", 1, 0.89f, 1.00f),
    XG_ENTRY(double, D_64x64x16, "d_64x64x16_w2x2", 4, 0.90f, 0.77f),
    XG_ENTRY(double, D_128x64x16, "d_128x64x16_w2x2", 3, 0.95f, 0.76f),
    XG_ENTRY(double, D_64x128x16, "d_64x128x16_w2x2", 3, 0.93f, 0.86f),
    XG_ENTRY(double, D_32x32x16, "d_32x32x16_w2x2", 8, 0.70f, 0.41f),
    };
    *n = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}

}  // namespace xg
