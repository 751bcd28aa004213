// xgemm_s.hip -- fp32 kernel instantiations (FP32 MFMA 32x32x2).
#include "tables.h"

namespace xg {

using S_128x128x16 = TileCfg<float, 128, 128, 16, 2, 2, 2>;
using S_256x128x16 = TileCfg<float, 256, 128, 16, 2, 2, 2>;
using S_64x64x16 = TileCfg<float, 64, 64, 16, 2, 2, 2>;
using S_128x128x32 = TileCfg<float, 128, 128, 32, 2, 2, 2>;

#define XG_ENTRY(T, CFG, NAME) {NAME, CFG::MT_M, CFG::MT_N, &launch_cfg<T, CFG>}

const VariantEntry<float> *s_variant_table(int *n) {
    static const VariantEntry<float> table[] = {
    XG_ENTRY(float, S_128x128x16, "s_128x128x16_w2x2"),
    XG_ENTRY(float, S_256x128x16, "s_256x128x16_w2x2"),
    XG_ENTRY(float, S_64x64x16, "s_64x64x16_w2x2"),
    XG_ENTRY(float, S_128x128x32, "s_128x128x32_w2x2"),
    };
    *n = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}

}  // namespace xg
