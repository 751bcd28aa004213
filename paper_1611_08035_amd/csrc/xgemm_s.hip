// xgemm_s.hip -- fp32 kernel instantiations (FP32 MFMA 32x32x2).
#include "tables.h"

namespace xg {

using S_128x128x16 = TileCfg<float, 128, 128, 16, 2, 2, 2>;
using S_256x128x16 = TileCfg<float, 256, 128, 16, 2, 2, 2>;
using S_64x64x16 = TileCfg<float, 64, 64, 16, 2, 2, 2, 2>;     // slabs asked for two ahead (a slab is shorter than a memory round trip)
using S_128x128x32 = TileCfg<float, 128, 128, 32, 2, 2, 2>;
using S_128x64x16 = TileCfg<float, 128, 64, 16, 2, 2, 2, 2>;   // the same

#define XG_ENTRY(T, CFG, NAME, WGS, EFF, LONE) {NAME, CFG::MT_M, CFG::MT_N, CFG::KT, CFG::WGM, CFG::WGN, WGS, EFF, LONE, false, &launch_cfg<T, CFG, false>}
// the same with the split-tail kernels built as well
#define XG_ENTRY_SPLIT(T, CFG, NAME, WGS, EFF, LONE) {NAME, CFG::MT_M, CFG::MT_N, CFG::KT, CFG::WGM, CFG::WGN, WGS, EFF, LONE, true, &launch_cfg<T, CFG, true>}

const VariantEntry<float> *s_variant_table(int *n) {
    static const VariantEntry<float> table[] = {
    XG_ENTRY_SPLIT(float, S_128x128x16, "s_128x128x16_w2x2", 2, 0.95f, 0.92f),
    XG_ENTRY_SPLIT(float, S_256x128x16, "s_256x128x16_w2x2", 2, 0.975f, 0.96f),
    XG_ENTRY(float, S_64x64x16, "s_64x64x16_w2x2", 4, 0.80f, 0.65f),
    XG_ENTRY(float, S_128x128x32, "s_128x128x32_w2x2", 2, 0.88f, 0.92f),
    XG_ENTRY(float, S_128x64x16, "s_128x64x16_w2x2", 3, 0.90f, 0.77f),
    };
    *n = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}

}  // namespace xg
